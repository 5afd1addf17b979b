// Mish, layer normalisation and softmax: HBM-bound operators, one pass over their tensors.
//
// Row-wise operators (layer normalisation, softmax): a wavefront owns a row.  The row lives in
// registers (NV float4 per lane, coalesced 1 KB per load instruction), so every statistic is a
// register pass plus a DPP wavefront reduction and the row is read from HBM exactly once (the
// paper's warp tiling with warp-level reductions, section "Softmax"; what depends on a
// reduction is recomputed from registers instead of being written out).  Rows longer than 2048
// take a workgroup per row with the row in LDS.  The weight gradients of layer normalisation
// are accumulated per lane over the rows a wavefront walks (a lane owns the same columns in
// every row), combined over the four wavefronts of a workgroup in LDS, written once per
// workgroup and added in a fixed order by a second stage: no atomics.
//
// Mish: forward y = x*t with t = tanh(softplus(x)) = n/(n+2), n = e^x*(e^x+2); backward
// recomputes t and sigmoid(x) from x alone, 1 - t^2 = w*(2-w) with w = 2/(n+2) (no
// cancellation).  16 bytes per lane, grid-stride.
#include "../../include/dnnops.h"
#include "mbconv_dev.h"
#include "mbconv_launch.h"

#include <mutex>

namespace mbk {
namespace {

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// ---- Mish ---------------------------------------------------------------------------------
__device__ __forceinline__ float mish_t(float x, float &w)
{
    // t = tanh(log(1+e^x)) = n/(n+2), w = 1 - t = 2/(n+2); beyond x = 20 the difference from 1
    // is below fp32 resolution and e^x*(e^x+2) would overflow
    const float e = __expf(fminf(x, 20.0f));
    const float n = e * (e + 2.0f);
    w = 2.0f * __builtin_amdgcn_rcpf(n + 2.0f);
    return 1.0f - w;
}
__device__ __forceinline__ float mish_val(float x)
{
    float w;
    return x * mish_t(x, w);
}
__device__ __forceinline__ float mish_grad(float x)
{
    float w;
    const float t = mish_t(x, w);
    const float s = sigmoidf_fast(x);
    return fmaf(x * s, w * (2.0f - w), t);
}

// Four 16-byte runs per thread and round, all loads of a round issued before the first use (a
// load-use-store loop would pay one memory round trip per run).
template <bool BWD>
__global__ __launch_bounds__(256) void mish_kernel(const float *__restrict__ x, const float *dy,
                                                   float *out, size_t n)
{
    constexpr int U = 4;
    const size_t n4 = n / 4;
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i0 = (size_t)blockIdx.x * 256 + threadIdx.x; i0 < n4; i0 += U * stride) {
        float4 xv[U], g[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t i = min(i0 + u * stride, n4 - 1); // clamped: always a valid run
            xv[u] = reinterpret_cast<const float4 *>(x)[i];
            if (BWD)
                g[u] = reinterpret_cast<const float4 *>(dy)[i];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float4 r;
            if (BWD)
                r = make_float4(g[u].x * mish_grad(xv[u].x), g[u].y * mish_grad(xv[u].y),
                                g[u].z * mish_grad(xv[u].z), g[u].w * mish_grad(xv[u].w));
            else
                r = make_float4(mish_val(xv[u].x), mish_val(xv[u].y), mish_val(xv[u].z), mish_val(xv[u].w));
            if (i0 + u * stride < n4)
                reinterpret_cast<float4 *>(out)[i0 + u * stride] = r;
        }
    }
    if (blockIdx.x == 0) { // at most three trailing elements
        const size_t i = 4 * n4 + threadIdx.x;
        if (i < n)
            out[i] = BWD ? dy[i] * mish_grad(x[i]) : mish_val(x[i]);
    }
}

// ---- rows in registers ------------------------------------------------------------------------
// Lane l, vector j covers columns 4*(l + 64*j) .. +3.  cols % 4 == 0, cols <= 256*NV.
template <int NV>
struct RowRegs {
    float v[NV][4];
    __device__ __forceinline__ void load(const float *row, int cols, int lane, float fill)
    {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = 4 * (lane + 64 * j);
            const float4 t = *reinterpret_cast<const float4 *>(row + min(c, cols - 4));
            const bool ok = c < cols;
            v[j][0] = ok ? t.x : fill;
            v[j][1] = ok ? t.y : fill;
            v[j][2] = ok ? t.z : fill;
            v[j][3] = ok ? t.w : fill;
        }
    }
    __device__ __forceinline__ void store(float *row, int cols, int lane) const
    {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = 4 * (lane + 64 * j);
            if (c < cols)
                *reinterpret_cast<float4 *>(row + c) = make_float4(v[j][0], v[j][1], v[j][2], v[j][3]);
        }
    }
};

template <int NV>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const float *__restrict__ x,
                                                            const float *__restrict__ gamma,
                                                            const float *__restrict__ beta, float eps,
                                                            int rows, int cols, float *y, float *mean,
                                                            float *rstd)
{
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = gridDim.x * 4;
    RowRegs<NV> g, b;
    g.load(gamma, cols, lane, 0.f);
    b.load(beta, cols, lane, 0.f);
    const float inv = 1.0f / (float)cols;
    for (int r = wave; r < rows; r += nwaves) {
        RowRegs<NV> a;
        a.load(x + (size_t)r * cols, cols, lane, 0.f);
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                s += a.v[j][k];
        const float mu = wave_sum(s) * inv;
        float s2 = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float d = (4 * (lane + 64 * j) < cols) ? a.v[j][k] - mu : 0.f;
                s2 = fmaf(d, d, s2);
            }
        const float rs = 1.0f / sqrtf(wave_sum(s2) * inv + eps);
#pragma unroll
        for (int j = 0; j < NV; ++j)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                a.v[j][k] = fmaf(g.v[j][k], (a.v[j][k] - mu) * rs, b.v[j][k]);
        a.store(y + (size_t)r * cols, cols, lane);
        if (lane == 0) {
            mean[r] = mu;
            rstd[r] = rs;
        }
    }
}

template <int NV>
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const float *__restrict__ x,
                                                            const float *__restrict__ dy,
                                                            const float *__restrict__ gamma,
                                                            const float *__restrict__ mean,
                                                            const float *__restrict__ rstd, int rows,
                                                            int cols, float *dx, float *pgamma,
                                                            float *pbeta)
{
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = gridDim.x * 4;
    RowRegs<NV> g, ag, ab;
    g.load(gamma, cols, lane, 0.f);
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int k = 0; k < 4; ++k)
            ag.v[j][k] = ab.v[j][k] = 0.f;
    const float inv = 1.0f / (float)cols;
    for (int r = wave; r < rows; r += nwaves) {
        RowRegs<NV> a, d;
        a.load(x + (size_t)r * cols, cols, lane, 0.f);
        d.load(dy + (size_t)r * cols, cols, lane, 0.f);
        const float mu = mean[r], rs = rstd[r];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float xh = (a.v[j][k] - mu) * rs; // padded columns: dy = 0 there
                const float gg = d.v[j][k] * g.v[j][k];
                ag.v[j][k] = fmaf(d.v[j][k], xh, ag.v[j][k]);
                ab.v[j][k] += d.v[j][k];
                a.v[j][k] = xh;
                d.v[j][k] = gg;
                s1 += gg;
                s2 = fmaf(gg, xh, s2);
            }
        const float m1 = wave_sum(s1) * inv, m2 = wave_sum(s2) * inv;
#pragma unroll
        for (int j = 0; j < NV; ++j)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                d.v[j][k] = rs * (d.v[j][k] - m1 - a.v[j][k] * m2);
        d.store(dx + (size_t)r * cols, cols, lane);
    }
    // one partial row per workgroup: the four wavefronts are added in a fixed order through LDS
    __shared__ float part[2][4][256 * NV];
    const int wv = threadIdx.x >> 6;
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            part[0][wv][4 * (lane + 64 * j) + k] = ag.v[j][k];
            part[1][wv][4 * (lane + 64 * j) + k] = ab.v[j][k];
        }
    __syncthreads();
    for (int c = threadIdx.x; c < cols; c += 256) {
        pgamma[(size_t)blockIdx.x * cols + c] = (part[0][0][c] + part[0][1][c]) + (part[0][2][c] + part[0][3][c]);
        pbeta[(size_t)blockIdx.x * cols + c] = (part[1][0][c] + part[1][1][c]) + (part[1][2][c] + part[1][3][c]);
    }
}

template <int NV, bool BWD>
__global__ __launch_bounds__(256) void softmax_kernel(const float *__restrict__ in0,
                                                      const float *__restrict__ in1, float *out,
                                                      int rows, int cols)
{
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = gridDim.x * 4;
    for (int r = wave; r < rows; r += nwaves) {
        RowRegs<NV> a;
        if (!BWD) {
            a.load(in0 + (size_t)r * cols, cols, lane, -INFINITY);
            float m = -INFINITY;
#pragma unroll
            for (int j = 0; j < NV; ++j)
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    m = fmaxf(m, a.v[j][k]);
            m = wave_max(m);
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < NV; ++j)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    a.v[j][k] = __expf(a.v[j][k] - m); // padded columns: exp(-inf) = 0
                    s += a.v[j][k];
                }
            const float is = 1.0f / wave_sum(s);
#pragma unroll
            for (int j = 0; j < NV; ++j)
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    a.v[j][k] *= is;
        } else {
            RowRegs<NV> d;
            a.load(in0 + (size_t)r * cols, cols, lane, 0.f); // y
            d.load(in1 + (size_t)r * cols, cols, lane, 0.f); // dy
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < NV; ++j)
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    s = fmaf(d.v[j][k], a.v[j][k], s);
            s = wave_sum(s);
#pragma unroll
            for (int j = 0; j < NV; ++j)
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    a.v[j][k] *= d.v[j][k] - s;
        }
        a.store(out + (size_t)r * cols, cols, lane);
    }
}

// ---- long or ragged rows: a workgroup per row, the row staged in LDS ----------------------------
// mode 0: layer-norm forward, 1: layer-norm backward (dx only; the column sums are taken by
// colsum_kernel), 2: softmax forward, 3: softmax backward.
__device__ __forceinline__ float block_reduce(float v, float *red, bool is_max)
{
    v = is_max ? wave_max(v) : wave_sum(v);
    __syncthreads(); // red may still be read from the previous reduction
    if ((threadIdx.x & 63) == 0)
        red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < 4; ++i)
        r = is_max ? fmaxf(r, red[i]) : r + red[i];
    return r;
}

template <int MODE>
__global__ __launch_bounds__(256) void row_generic_kernel(const float *__restrict__ in0,
                                                          const float *__restrict__ in1,
                                                          const float *__restrict__ gamma,
                                                          const float *__restrict__ beta, float eps,
                                                          int rows, int cols, float *out, float *mean,
                                                          float *rstd)
{
    extern __shared__ float rowbuf[]; // [cols] (+ [cols] for the two-input modes)
    __shared__ float red[4];
    const int tid = threadIdx.x;
    const float inv = 1.0f / (float)cols;
    for (int r = blockIdx.x; r < rows; r += gridDim.x) {
        const size_t o = (size_t)r * cols;
        __syncthreads(); // the previous row's buffer has been consumed
        for (int c = tid; c < cols; c += 256) {
            rowbuf[c] = in0[o + c];
            if (MODE == 1 || MODE == 3)
                rowbuf[cols + c] = in1[o + c];
        }
        __syncthreads();
        if (MODE == 0) {
            float s = 0.f;
            for (int c = tid; c < cols; c += 256)
                s += rowbuf[c];
            const float mu = block_reduce(s, red, false) * inv;
            float s2 = 0.f;
            for (int c = tid; c < cols; c += 256)
                s2 = fmaf(rowbuf[c] - mu, rowbuf[c] - mu, s2);
            const float rs = 1.0f / sqrtf(block_reduce(s2, red, false) * inv + eps);
            for (int c = tid; c < cols; c += 256)
                out[o + c] = fmaf(gamma[c], (rowbuf[c] - mu) * rs, beta[c]);
            if (tid == 0) {
                mean[r] = mu;
                rstd[r] = rs;
            }
        } else if (MODE == 1) { // in0 = x, in1 = dy
            const float mu = mean[r], rs = rstd[r];
            float s1 = 0.f, s2 = 0.f;
            for (int c = tid; c < cols; c += 256) {
                const float gg = rowbuf[cols + c] * gamma[c];
                s1 += gg;
                s2 = fmaf(gg, (rowbuf[c] - mu) * rs, s2);
            }
            const float m1 = block_reduce(s1, red, false) * inv;
            const float m2 = block_reduce(s2, red, false) * inv;
            for (int c = tid; c < cols; c += 256)
                out[o + c] = rs * (rowbuf[cols + c] * gamma[c] - m1 - (rowbuf[c] - mu) * rs * m2);
        } else if (MODE == 2) {
            float m = -INFINITY;
            for (int c = tid; c < cols; c += 256)
                m = fmaxf(m, rowbuf[c]);
            m = block_reduce(m, red, true);
            float s = 0.f;
            for (int c = tid; c < cols; c += 256) {
                const float e = __expf(rowbuf[c] - m);
                rowbuf[c] = e; // each thread rewrites only its own columns
                s += e;
            }
            const float is = 1.0f / block_reduce(s, red, false);
            for (int c = tid; c < cols; c += 256)
                out[o + c] = rowbuf[c] * is;
        } else { // in0 = y, in1 = dy
            float s = 0.f;
            for (int c = tid; c < cols; c += 256)
                s = fmaf(rowbuf[cols + c], rowbuf[c], s);
            s = block_reduce(s, red, false);
            for (int c = tid; c < cols; c += 256)
                out[o + c] = rowbuf[c] * (rowbuf[cols + c] - s);
        }
    }
}

// Column sums for the generic layer-norm backward: workgroup (column block of 64, row slice)
// writes partial[slice][cols] for dgamma and dbeta; rows are added in ascending order.
__global__ __launch_bounds__(256) void ln_colsum_kernel(const float *__restrict__ x,
                                                        const float *__restrict__ dy,
                                                        const float *__restrict__ mean,
                                                        const float *__restrict__ rstd, int rows,
                                                        int cols, int rowsPerSlice, float *pgamma,
                                                        float *pbeta)
{
    __shared__ float red[2][4][64];
    const int c = blockIdx.x * 64 + (threadIdx.x & 63), q = threadIdx.x >> 6;
    const int r0 = blockIdx.y * rowsPerSlice, r1 = min(r0 + rowsPerSlice, rows);
    float sg = 0.f, sb = 0.f;
    if (c < cols)
        for (int r = r0 + q; r < r1; r += 4) {
            const float d = dy[(size_t)r * cols + c];
            sg = fmaf(d, (x[(size_t)r * cols + c] - mean[r]) * rstd[r], sg);
            sb += d;
        }
    red[0][q][threadIdx.x & 63] = sg;
    red[1][q][threadIdx.x & 63] = sb;
    __syncthreads();
    if (q == 0 && c < cols) {
        const int l = threadIdx.x;
        pgamma[(size_t)blockIdx.y * cols + c] = (red[0][0][l] + red[0][1][l]) + (red[0][2][l] + red[0][3][l]);
        pbeta[(size_t)blockIdx.y * cols + c] = (red[1][0][l] + red[1][1][l]) + (red[1][2][l] + red[1][3][l]);
    }
}

// ---- host side ----------------------------------------------------------------------------------
bool bad_align(const void *p) { return ((uintptr_t)p & 15u) != 0; }

// rows in registers: cols % 4 == 0 and cols <= 2048
int row_nv(int cols)
{
    if (cols % 4 != 0 || cols > 2048)
        return 0;
    return cols <= 256 ? 1 : cols <= 512 ? 2 : cols <= 1024 ? 4 : 8;
}
int row_grid(int rows) // four rows per workgroup in flight, at most 2048 workgroups
{
    const int g = (rows + 3) / 4;
    return g < 1 ? 1 : (g > 2048 ? 2048 : g);
}
int row_grid_bwd(int rows) // sixteen rows per workgroup, at most 512 partial rows
{
    const int g = (rows + 15) / 16;
    return g < 1 ? 1 : (g > 512 ? 512 : g);
}
int generic_grid(int rows) { return rows > 4096 ? 4096 : rows; }
int ln_slices(int rows) // row slices of the generic column sums
{
    const int s = (rows + 63) / 64;
    return s > 256 ? 256 : (s < 1 ? 1 : s);
}

} // namespace
} // namespace mbk

using namespace mbk;

// ---- scratch for callers that cannot allocate --------------------------------------------------
// dnnops_layernorm_backward_noalloc keeps the partial sums of the two weight gradients in this
// array instead of a caller's workspace.  One copy exists on every GPU the library runs on, from
// the time the code object is loaded until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress: the device address is looked up once per device, with
// that device current, and kept in g_ln_scratch_ptr; kernels and the second stage receive that
// address as an ordinary pointer argument.
#define DNNOPS_STATIC_SCRATCH_BYTES (8u << 20)
static __device__ __align__(256) unsigned char ln_static_scratch[DNNOPS_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_ln_scratch_mutex;
void *g_ln_scratch_ptr[kMaxDevices] = {};

// Device address of this GPU's copy of ln_static_scratch (nullptr on failure).
void *ln_static_scratch_ptr()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return nullptr;
    std::lock_guard<std::mutex> lock(g_ln_scratch_mutex);
    if (!g_ln_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(ln_static_scratch)) != hipSuccess || !ptr)
            return nullptr;
        g_ln_scratch_ptr[dev] = ptr;
    }
    return g_ln_scratch_ptr[dev];
}
} // namespace

extern "C" {

dnnops_status dnnops_mish_forward(const float *x, float *y, size_t n, void *hip_stream)
{
    if (!x || !y || n == 0)
        return DNNOPS_EINVAL;
    if (bad_align(x) || bad_align(y))
        return DNNOPS_EALIGN;
    const size_t wg = (n / 4 + 1023) / 1024; // four runs per thread
    const unsigned grid = (unsigned)(wg < 1 ? 1 : (wg > 65536 ? 65536 : wg));
    hipLaunchKernelGGL(mish_kernel<false>, dim3(grid), dim3(256), 0, (hipStream_t)hip_stream, x,
                       (const float *)nullptr, y, n);
    return hipGetLastError() == hipSuccess ? DNNOPS_OK : DNNOPS_EHIP;
}

dnnops_status dnnops_mish_backward(const float *x, const float *dy, float *dx, size_t n,
                                   void *hip_stream)
{
    if (!x || !dy || !dx || n == 0)
        return DNNOPS_EINVAL;
    if (bad_align(x) || bad_align(dy) || bad_align(dx))
        return DNNOPS_EALIGN;
    const size_t wg = (n / 4 + 1023) / 1024;
    const unsigned grid = (unsigned)(wg < 1 ? 1 : (wg > 65536 ? 65536 : wg));
    hipLaunchKernelGGL(mish_kernel<true>, dim3(grid), dim3(256), 0, (hipStream_t)hip_stream, x, dy,
                       dx, n);
    return hipGetLastError() == hipSuccess ? DNNOPS_OK : DNNOPS_EHIP;
}

#define DNNOPS_NV_SWITCH(nv, CALL)                                                                \
    switch (nv) {                                                                                 \
    case 1: { constexpr int NV = 1; CALL; } break;                                                \
    case 2: { constexpr int NV = 2; CALL; } break;                                                \
    case 4: { constexpr int NV = 4; CALL; } break;                                                \
    default: { constexpr int NV = 8; CALL; } break;                                               \
    }

dnnops_status dnnops_layernorm_forward(const float *x, const float *gamma, const float *beta,
                                       float eps, int32_t rows, int32_t cols, float *y, float *mean,
                                       float *rstd, void *hip_stream)
{
    if (!x || !gamma || !beta || !y || !mean || !rstd || rows < 1 || cols < 1 || !(eps >= 0.f))
        return DNNOPS_EINVAL;
    if (cols > DNNOPS_MAX_COLS)
        return DNNOPS_EUNSUPPORTED;
    if (bad_align(x) || bad_align(gamma) || bad_align(beta) || bad_align(y))
        return DNNOPS_EALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    const int nv = row_nv(cols);
    if (nv) {
        DNNOPS_NV_SWITCH(nv, hipLaunchKernelGGL((layernorm_fwd_kernel<NV>), dim3(row_grid(rows)), dim3(256),
                                                0, st, x, gamma, beta, eps, rows, cols, y, mean, rstd));
    } else {
        hipLaunchKernelGGL((row_generic_kernel<0>), dim3(generic_grid(rows)), dim3(256),
                           sizeof(float) * cols, st, x, (const float *)nullptr, gamma, beta, eps, rows,
                           cols, y, mean, rstd);
    }
    return hipGetLastError() == hipSuccess ? DNNOPS_OK : DNNOPS_EHIP;
}

size_t dnnops_layernorm_backward_scratch_bytes(int32_t rows, int32_t cols)
{
    if (rows < 1 || cols < 1 || cols > DNNOPS_MAX_COLS)
        return 0;
    const size_t parts = row_nv(cols) ? (size_t)row_grid_bwd(rows) : (size_t)ln_slices(rows);
    return 2 * parts * (size_t)cols * sizeof(float);
}

static dnnops_status layernorm_backward_check(const float *x, const float *dy, const float *gamma,
                                              const float *mean, const float *rstd, int32_t rows,
                                              int32_t cols, float *dx, float *dgamma, float *dbeta)
{
    if (!x || !dy || !gamma || !mean || !rstd || !dx || !dgamma || !dbeta || rows < 1 || cols < 1)
        return DNNOPS_EINVAL;
    if (cols > DNNOPS_MAX_COLS)
        return DNNOPS_EUNSUPPORTED;
    if (bad_align(x) || bad_align(dy) || bad_align(gamma) || bad_align(dx))
        return DNNOPS_EALIGN;
    return DNNOPS_OK;
}

// Both entry points: dx and the per-workgroup partial sums of dgamma, dbeta into `scratch`, then
// their fixed-order sum.  Every partial the second stage reads is written by the first.
static dnnops_status layernorm_backward_launch(const float *x, const float *dy, const float *gamma,
                                               const float *mean, const float *rstd, int32_t rows,
                                               int32_t cols, float *dx, float *dgamma, float *dbeta,
                                               void *scratch, hipStream_t st)
{
    const int nv = row_nv(cols);
    int parts;
    float *pg = (float *)scratch;
    if (nv) {
        parts = row_grid_bwd(rows);
        float *pb = pg + (size_t)parts * cols;
        DNNOPS_NV_SWITCH(nv, hipLaunchKernelGGL((layernorm_bwd_kernel<NV>), dim3(parts), dim3(256),
                                                0, st, x, dy, gamma, mean, rstd, rows, cols, dx, pg, pb));
    } else {
        parts = ln_slices(rows);
        float *pb = pg + (size_t)parts * cols;
        hipLaunchKernelGGL((row_generic_kernel<1>), dim3(generic_grid(rows)), dim3(256),
                           2 * sizeof(float) * cols, st, x, dy, gamma, (const float *)nullptr, 0.f,
                           rows, cols, dx, const_cast<float *>(mean), const_cast<float *>(rstd));
        const int per = (rows + parts - 1) / parts;
        hipLaunchKernelGGL(ln_colsum_kernel, dim3((cols + 63) / 64, parts), dim3(256), 0, st, x, dy,
                           mean, rstd, rows, cols, per, pg, pb);
    }
    if (hipGetLastError() != hipSuccess)
        return DNNOPS_EHIP;
    float *pb = pg + (size_t)parts * cols;
    if (launch_reduce_splits2({pg, parts, (size_t)cols, dgamma}, {pb, parts, (size_t)cols, dbeta}, st) !=
        hipSuccess)
        return DNNOPS_EHIP;
    return DNNOPS_OK;
}

dnnops_status dnnops_layernorm_backward(const float *x, const float *dy, const float *gamma,
                                        const float *mean, const float *rstd, int32_t rows,
                                        int32_t cols, float *dx, float *dgamma, float *dbeta,
                                        void *scratch, void *hip_stream)
{
    if (!scratch)
        return DNNOPS_EINVAL;
    const dnnops_status s = layernorm_backward_check(x, dy, gamma, mean, rstd, rows, cols, dx, dgamma, dbeta);
    if (s != DNNOPS_OK)
        return s;
    if (bad_align(scratch))
        return DNNOPS_EALIGN;
    return layernorm_backward_launch(x, dy, gamma, mean, rstd, rows, cols, dx, dgamma, dbeta, scratch,
                                     (hipStream_t)hip_stream);
}

size_t dnnops_layernorm_backward_noalloc_max_scratch_bytes(void) { return DNNOPS_STATIC_SCRATCH_BYTES; }

dnnops_status dnnops_layernorm_backward_noalloc(const float *x, const float *dy, const float *gamma,
                                                const float *mean, const float *rstd, int32_t rows,
                                                int32_t cols, float *dx, float *dgamma,
                                                float *dbeta, void *hip_stream)
{
    const dnnops_status s = layernorm_backward_check(x, dy, gamma, mean, rstd, rows, cols, dx, dgamma, dbeta);
    if (s != DNNOPS_OK)
        return s;
    // host-side size check ahead of any HIP call
    if (dnnops_layernorm_backward_scratch_bytes(rows, cols) > DNNOPS_STATIC_SCRATCH_BYTES)
        return DNNOPS_ESCRATCH;
    void *scratch = ln_static_scratch_ptr();
    if (!scratch)
        return DNNOPS_EHIP;
    return layernorm_backward_launch(x, dy, gamma, mean, rstd, rows, cols, dx, dgamma, dbeta, scratch,
                                     (hipStream_t)hip_stream);
}

static dnnops_status softmax_launch(bool bwd, const float *in0, const float *in1, float *out,
                                    int32_t rows, int32_t cols, void *hip_stream)
{
    if (!in0 || (bwd && !in1) || !out || rows < 1 || cols < 1)
        return DNNOPS_EINVAL;
    if (cols > DNNOPS_MAX_COLS)
        return DNNOPS_EUNSUPPORTED;
    if (bad_align(in0) || bad_align(in1) || bad_align(out))
        return DNNOPS_EALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    const int nv = row_nv(cols);
    if (nv) {
        if (bwd) {
            DNNOPS_NV_SWITCH(nv, hipLaunchKernelGGL((softmax_kernel<NV, true>), dim3(row_grid(rows)),
                                                    dim3(256), 0, st, in0, in1, out, rows, cols));
        } else {
            DNNOPS_NV_SWITCH(nv, hipLaunchKernelGGL((softmax_kernel<NV, false>), dim3(row_grid(rows)),
                                                    dim3(256), 0, st, in0, in1, out, rows, cols));
        }
    } else if (bwd) {
        hipLaunchKernelGGL((row_generic_kernel<3>), dim3(generic_grid(rows)), dim3(256),
                           2 * sizeof(float) * cols, st, in0, in1, (const float *)nullptr,
                           (const float *)nullptr, 0.f, rows, cols, out, (float *)nullptr,
                           (float *)nullptr);
    } else {
        hipLaunchKernelGGL((row_generic_kernel<2>), dim3(generic_grid(rows)), dim3(256),
                           sizeof(float) * cols, st, in0, in1, (const float *)nullptr,
                           (const float *)nullptr, 0.f, rows, cols, out, (float *)nullptr,
                           (float *)nullptr);
    }
    return hipGetLastError() == hipSuccess ? DNNOPS_OK : DNNOPS_EHIP;
}

dnnops_status dnnops_softmax_forward(const float *x, float *y, int32_t rows, int32_t cols,
                                     void *hip_stream)
{
    return softmax_launch(false, x, nullptr, y, rows, cols, hip_stream);
}

dnnops_status dnnops_softmax_backward(const float *y, const float *dy, float *dx, int32_t rows,
                                      int32_t cols, void *hip_stream)
{
    return softmax_launch(true, y, dy, dx, rows, cols, hip_stream);
}

} // extern "C"
