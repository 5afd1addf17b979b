// Register-direct 1x1 convolutions and weight gradients for the HBM-bound ("skinny") shapes.
//
// When one side of the 1x1 convolution has few channels (the 24 <-> 144 pairs of the early
// EfficientNet stages) the GEMM moves far more bytes than it has flops to hide them behind,
// so the kernels below are built around the memory system of gfx950: every global access is
// 16 bytes per lane (a dword-per-lane stream reaches under half the bandwidth of a 16-byte
// one on this chip), activations never pass through LDS, and there is no barrier in a main
// loop.
//
// MFMA used: v_mfma_f32_32x32x2_f32, C[i][j] += sum_k A[i][k]*B[k][j] with
//   A: lane l holds A[i = l%32][k = l/32],  B: lane l holds B[k = l/32][j = l%32],
//   C: lane l, register r holds C[i = 8*(r/4) + 4*(l/32) + r%4][j = l%32].
//
// conv_ce / conv_cr (forward convs and data gradients), "pixel-vector" form:
//   out[ch][pix] = sum_k W[ch][k] * act[k][pix].  A = weights (i = output channel), B =
//   activations (j = pixel).  A lane loads FOUR consecutive pixels of one input channel
//   (float4; a wavefront covers 2 channels x 128 pixels per load) and feeds element r of the
//   vector to MFMA number r, so four accumulator tiles C_r cover pixels 4j+r.  Register q of
//   the four tiles is then again four consecutive pixels of one output channel: the stores are
//   float4 too, 512 contiguous bytes per output-channel row.
//   - conv_ce (few input channels, K <= 40): one wavefront per 32-output-channel tile, the
//     whole activation tile in registers.
//   - conv_cr (few output channels, M <= 64): the input channels are split over the four
//     wavefronts of the workgroup (each matrix core gets a quarter of the MFMAs), partial
//     accumulators are exchanged through LDS once per tile.
//   The elementwise prologues (Swish(BN(.))*gate, BN backward) run on the activation
//   registers between load and MFMA, so those tensors never exist in memory (recomputation
//   instead of load/store: section "Backpropagation and Data Movement" of the paper).
//
// wgrad_cl (weight gradients), "channel-lane" form: dW[a][b] = sum_pix U[a][pix]*V[b][pix].
//   The contraction runs over pixels, so a lane owns a channel (A: i = a, B: j = b) and loads
//   float4 runs of its channel's pixels; the two lane halves and the four vector elements
//   enumerate the contraction index.  Workgroups split the pixel range; partial tiles are
//   summed in a fixed order by reduce_splits (no atomics: the paper's map-fission step,
//   section "Guided Optimization Case Study: EfficientNet").
#include "mbconv_dev.h"
#include "mbconv_launch.h"

namespace mbk {

typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));

struct WaveConvArgs {
    int N, M, K, HW;
    uint32_t Q; // N*HW, a multiple of 4
    int numTiles;
    FastDiv divHW;
    const void *w;
    int sAm, sAk;
    const void *p0, *p1;
    const float *c0, *c1, *c2, *gate;
    void *out;
    const void *res;
    float *psum, *psq;
    int NP; // partial-sum slots per channel (= gridDim.x)
};

template <typename T>
__device__ __forceinline__ void store4(T *p, size_t i, const float (&v)[4]);
template <>
__device__ __forceinline__ void store4<float>(float *p, size_t i, const float (&v)[4])
{
    float4v t = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<float4v *>(p + i) = t;
}
template <>
__device__ __forceinline__ void store4<bf16_t>(bf16_t *p, size_t i, const float (&v)[4])
{
    uint2 t;
    t.x = (uint32_t)float_to_bf16_bits(v[0]) | ((uint32_t)float_to_bf16_bits(v[1]) << 16);
    t.y = (uint32_t)float_to_bf16_bits(v[2]) | ((uint32_t)float_to_bf16_bits(v[3]) << 16);
    *reinterpret_cast<uint2 *>(&p[i]) = t;
}

template <typename T>
__device__ __forceinline__ void load4(const T *p, size_t i, float (&v)[4]);
template <>
__device__ __forceinline__ void load4<float>(const float *p, size_t i, float (&v)[4])
{
    const float4v t = *reinterpret_cast<const float4v *>(p + i);
    v[0] = t.x;
    v[1] = t.y;
    v[2] = t.z;
    v[3] = t.w;
}
template <>
__device__ __forceinline__ void load4<bf16_t>(const bf16_t *p, size_t i, float (&v)[4])
{
    const uint2 t = *reinterpret_cast<const uint2 *>(&p[i]);
    v[0] = bf16_bits_to_float(t.x & 0xffffu);
    v[1] = bf16_bits_to_float(t.x >> 16);
    v[2] = bf16_bits_to_float(t.y & 0xffffu);
    v[3] = bf16_bits_to_float(t.y >> 16);
}

// Prologue of one float4 of activations of input channel k, image n (see PRO_* in the header).
template <typename T, int PRO>
__device__ __forceinline__ void load_act4(const WaveConvArgs &a, size_t idx, uint32_t n, int k,
                                          const float *coef, int cstride, float (&v)[4])
{
    load4<T>((const T *)a.p0, idx, v);
    if (PRO == PRO_BNBWD) {
        float raw[4];
        load4<T>((const T *)a.p1, idx, raw);
        const float c0 = coef[k], c1 = coef[cstride + k], c2 = coef[2 * cstride + k];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            v[r] = fmaf(c0, v[r], fmaf(c1, raw[r], c2));
    } else if (PRO == PRO_BNSWISH_GATE) {
        const float sc = coef[k], sh = coef[cstride + k];
        const float g = a.gate[(size_t)n * a.K + k];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            v[r] = swishf(fmaf(v[r], sc, sh)) * g;
    }
}

template <int PRO>
__device__ __forceinline__ void stage_coef(const WaveConvArgs &a, float *coef, int cstride)
{
    if (PRO == PRO_NONE)
        return;
    for (int idx = threadIdx.x; idx < cstride; idx += blockDim.x) {
        const bool ok = idx < a.K;
        coef[idx] = ok ? a.c0[idx] : 0.f;
        coef[cstride + idx] = ok ? a.c1[idx] : 0.f;
        if (PRO == PRO_BNBWD)
            coef[2 * cstride + idx] = ok ? a.c2[idx] : 0.f;
    }
}

// ---- conv_ce: few input channels -------------------------------------------------------------
constexpr int kCeMaxMT = 8;

// blockDim = 64 * ceil(M/32); wavefront t produces output channels [32t, 32t+32).
template <typename T, int KS, int PRO, int EPI>
__global__ __launch_bounds__(64 * kCeMaxMT) void conv_ce_kernel(WaveConvArgs a)
{
    __shared__ float coef[3 * 2 * KS];
    __shared__ float red[kCeMaxMT][2][32];
    const int lane = threadIdx.x & 63, t = threadIdx.x >> 6;
    const int h = lane >> 5, j = lane & 31;
    stage_coef<PRO>(a, coef, 2 * KS);

    // this wavefront's weights, in A-operand order, straight into registers
    float wreg[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        const int m = 32 * t + j, k = 2 * s + h;
        wreg[s] = (m < a.M && k < a.K)
                      ? ld<T>((const T *)a.w, (size_t)m * a.sAm + (size_t)k * a.sAk)
                      : 0.f;
    }
    if (PRO != PRO_NONE)
        __syncthreads();

    float ssum[16], ssq[16];
#pragma unroll
    for (int q = 0; q < 16; ++q)
        ssum[q] = ssq[q] = 0.f;

    for (int tile = blockIdx.x; tile < a.numTiles; tile += gridDim.x) {
        const uint32_t qv = (uint32_t)tile * 128u + 4u * j;
        const bool valid = qv < a.Q;
        const uint32_t n = valid ? fdiv(qv, a.divHW) : 0;
        const uint32_t pix = valid ? qv - n * (uint32_t)a.HW : 0;
        float bv[KS][4];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int k = 2 * s + h;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                bv[s][r] = 0.f;
            if (valid && k < a.K)
                load_act4<T, PRO>(a, ((size_t)n * a.K + k) * a.HW + pix, n, k, coef, 2 * KS, bv[s]);
        }
        float16v acc[4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            acc[r] = (float16v){0};
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                acc[r] = __builtin_amdgcn_mfma_f32_32x32x2f32(wreg[s], bv[s][r], acc[r], 0, 0, 0);
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int m = 32 * t + 8 * (q >> 2) + 4 * h + (q & 3);
            if (valid && m < a.M) {
                const size_t idx = ((size_t)n * a.M + m) * a.HW + pix;
                float v[4] = {acc[0][q], acc[1][q], acc[2][q], acc[3][q]};
                if (EPI == EPI_RES) {
                    float rr[4];
                    load4<T>((const T *)a.res, idx, rr);
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        v[r] += rr[r];
                }
                store4<T>((T *)a.out, idx, v);
                if (EPI == EPI_STATS) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float sv = as_stored<T>(v[r]);
                        ssum[q] += sv;
                        ssq[q] = fmaf(sv, sv, ssq[q]);
                    }
                }
            }
        }
    }
    if (EPI == EPI_STATS) {
        // register q of the lanes that share l/32 belongs to one channel: sum over those 32 lanes
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const float s = half_wave_sum(ssum[q]);
            const float s2 = half_wave_sum(ssq[q]);
            if (j == 0) {
                const int row = 8 * (q >> 2) + 4 * h + (q & 3);
                red[t][0][row] = s;
                red[t][1][row] = s2;
            }
        }
        __syncthreads();
        if (lane < 32) {
            const int m = 32 * t + lane;
            if (m < a.M) {
                a.psum[(size_t)m * a.NP + blockIdx.x] = red[t][0][lane];
                a.psq[(size_t)m * a.NP + blockIdx.x] = red[t][1][lane];
            }
        }
    }
}

// ---- conv_cr: few output channels --------------------------------------------------------------
// 4 wavefronts; wavefront w contracts input-channel pairs [w*KSW, (w+1)*KSW).  After the
// contraction every wavefront holds a partial 32 x 128 output tile per channel tile; register
// group [4g, 4g+4) of it goes to wavefront g, which adds the four partials in wavefront order
// and finishes those output channels (8g + 4*(l/32) + 0..3 of the tile).
template <typename T, int MTS, int PRO, int EPI>
__global__ __launch_bounds__(256) void conv_cr_kernel(WaveConvArgs a)
{
    extern __shared__ float lds[];
    const int KS = (a.K + 1) >> 1;
    const int KSW = (KS + 3) >> 2;
    float *wl = lds;                          // [KS][MTS][64] A-operand order
    float *coef = wl + KS * MTS * 64;         // [3][2*KS]
    float *xch = coef + 6 * KS;               // [4 src][3 other dst][MTS*16 values][64 lanes]
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int h = lane >> 5, j = lane & 31;
    for (int idx = threadIdx.x; idx < KS * MTS * 64; idx += 256) {
        const int ln = idx & 63, st_ = idx >> 6;
        const int tt = st_ % MTS, s = st_ / MTS;
        const int m = 32 * tt + (ln & 31), k = 2 * s + (ln >> 5);
        wl[idx] = (m < a.M && k < a.K)
                      ? ld<T>((const T *)a.w, (size_t)m * a.sAm + (size_t)k * a.sAk)
                      : 0.f;
    }
    stage_coef<PRO>(a, coef, 2 * KS);
    __syncthreads();

    float ssum[MTS][4], ssq[MTS][4];
#pragma unroll
    for (int tt = 0; tt < MTS; ++tt)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            ssum[tt][i] = ssq[tt][i] = 0.f;

    const int sBeg = w * KSW, sEnd = (sBeg + KSW < KS) ? sBeg + KSW : KS;
    constexpr int U = 6; // channel pairs loaded per batch

    for (int tile = blockIdx.x; tile < a.numTiles; tile += gridDim.x) {
        const uint32_t qv = (uint32_t)tile * 128u + 4u * j;
        const bool valid = qv < a.Q;
        const uint32_t n = valid ? fdiv(qv, a.divHW) : 0;
        const uint32_t pix = valid ? qv - n * (uint32_t)a.HW : 0;
        const size_t base = (size_t)n * a.K * a.HW + pix;
        float16v acc[MTS][4];
#pragma unroll
        for (int tt = 0; tt < MTS; ++tt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                acc[tt][r] = (float16v){0};

        for (int s0 = sBeg; s0 < sEnd; s0 += U) {
            float bv[U][4];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int s = s0 + u, k = 2 * s + h;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    bv[u][r] = 0.f;
                if (valid && s < sEnd && k < a.K)
                    load_act4<T, PRO>(a, base + (size_t)k * a.HW, n, k, coef, 2 * KS, bv[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int s = s0 + u;
                if (s < sEnd) {
#pragma unroll
                    for (int tt = 0; tt < MTS; ++tt) {
                        const float wv = wl[(s * MTS + tt) * 64 + lane];
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            acc[tt][r] = __builtin_amdgcn_mfma_f32_32x32x2f32(wv, bv[u][r],
                                                                              acc[tt][r], 0, 0, 0);
                    }
                }
            }
        }
        // exchange: value (tt,i,r) of register group g goes to wavefront g; a wavefront keeps
        // its own group in registers and uses slot src*3 + (dst - (dst > src)) for the others
        float own[MTS][4][4];
        __syncthreads(); // previous tile's exchange buffer fully consumed
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if (g == w) {
#pragma unroll
                for (int tt = 0; tt < MTS; ++tt)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            own[tt][i][r] = acc[tt][r][4 * g + i];
            } else {
                const int slot = w * 3 + (g < w ? g : g - 1);
#pragma unroll
                for (int tt = 0; tt < MTS; ++tt)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            xch[((slot * (MTS * 16)) + (tt * 4 + i) * 4 + r) * 64 + lane] =
                                acc[tt][r][4 * g + i];
            }
        }
        __syncthreads();
#pragma unroll
        for (int tt = 0; tt < MTS; ++tt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float sacc = 0.f;
#pragma unroll
                    for (int src = 0; src < 4; ++src) {
                        if (src == w) {
                            sacc += own[tt][i][r];
                        } else {
                            const int slot = src * 3 + (w < src ? w : w - 1);
                            sacc += xch[((slot * (MTS * 16)) + (tt * 4 + i) * 4 + r) * 64 + lane];
                        }
                    }
                    v[r] = sacc;
                }
                const int m = 32 * tt + 8 * w + 4 * h + i;
                if (valid && m < a.M) {
                    const size_t idx = ((size_t)n * a.M + m) * a.HW + pix;
                    if (EPI == EPI_RES) {
                        float rr[4];
                        load4<T>((const T *)a.res, idx, rr);
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            v[r] += rr[r];
                    }
                    store4<T>((T *)a.out, idx, v);
                    if (EPI == EPI_STATS) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const float sv = as_stored<T>(v[r]);
                            ssum[tt][i] += sv;
                            ssq[tt][i] = fmaf(sv, sv, ssq[tt][i]);
                        }
                    }
                }
            }
    }
    if (EPI == EPI_STATS) {
#pragma unroll
        for (int tt = 0; tt < MTS; ++tt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float s = half_wave_sum(ssum[tt][i]);
                const float s2 = half_wave_sum(ssq[tt][i]);
                const int m = 32 * tt + 8 * w + 4 * h + i;
                if (j == 0 && m < a.M) {
                    a.psum[(size_t)m * a.NP + blockIdx.x] = s;
                    a.psq[(size_t)m * a.NP + blockIdx.x] = s2;
                }
            }
    }
}

// ---- dispatch of the two convolutions ---------------------------------------------------------

// conv_ce ends with a cross-lane reduction of its statistics, so it gets few workgroups that
// each take several tiles; conv_cr has one short tile per workgroup.
static int wave_conv_grid(int kind, int numTiles)
{
    const int cap = kind == 1 ? 264 : 2048;
    return numTiles < cap ? numTiles : cap;
}

static size_t conv_cr_lds(int M, int K)
{
    const int ks = (K + 1) / 2, mts = (M + 31) / 32;
    return sizeof(float) * ((size_t)ks * mts * 64 + 6 * ks + (size_t)12 * mts * 16 * 64);
}

// Which register-direct kernel covers (M, K, HW), if any: 1 = conv_ce, 2 = conv_cr, 0 = none.
int wave_conv_kind(int M, int K, int HW)
{
    if (HW % 4 != 0)
        return 0;
    if (K <= 40 && M <= 32 * kCeMaxMT)
        return 1;
    if (M <= 64 && conv_cr_lds(M, K) <= 150 * 1024)
        return 2;
    return 0;
}

int wave_conv_num_partials(int kind, int N, int HW)
{
    return wave_conv_grid(kind, (int)(((long long)N * HW + 127) / 128));
}

template <typename T, int PRO, int EPI>
static hipError_t launch_ce(const WaveConvArgs &a, int grid, hipStream_t st)
{
    const int ks = (a.K + 1) / 2, MT = (a.M + 31) / 32;
#define MBK_E(KS)                                                                                 \
    if (ks <= KS) {                                                                               \
        hipLaunchKernelGGL((conv_ce_kernel<T, KS, PRO, EPI>), dim3(grid), dim3(64 * MT), 0, st, a); \
        return hipGetLastError();                                                                 \
    }
    MBK_E(8)
    MBK_E(12)
    MBK_E(16)
    MBK_E(20)
#undef MBK_E
    return hipErrorInvalidValue;
}

template <typename T, int PRO, int EPI>
static hipError_t launch_cr(const WaveConvArgs &a, int grid, hipStream_t st)
{
    const int mts = (a.M + 31) / 32;
    const size_t lds = conv_cr_lds(a.M, a.K);
#define MBK_R(MTS)                                                                                \
    if (mts == MTS) {                                                                             \
        auto kern = conv_cr_kernel<T, MTS, PRO, EPI>;                                             \
        hipError_t e = hipFuncSetAttribute((const void *)kern,                                    \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess)                                                                      \
            return e;                                                                             \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, a);                              \
        return hipGetLastError();                                                                 \
    }
    MBK_R(1)
    MBK_R(2)
#undef MBK_R
    return hipErrorInvalidValue;
}

template <typename T>
static hipError_t wave_dispatch(const WaveConvArgs &a, int kind, int pro, int epi, int grid,
                                hipStream_t st)
{
#define MBK_CASE(P, E)                                                                            \
    if (pro == P && epi == E)                                                                     \
        return kind == 1 ? launch_ce<T, P, E>(a, grid, st) : launch_cr<T, P, E>(a, grid, st);
    MBK_CASE(PRO_NONE, EPI_STATS)
    MBK_CASE(PRO_BNSWISH_GATE, EPI_STATS)
    MBK_CASE(PRO_BNBWD, EPI_NONE)
    MBK_CASE(PRO_BNBWD, EPI_RES)
#undef MBK_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_wave_conv1x1(bool bf16, int kind, int N, int M, int K, int HW, const void *w,
                               int sAm, int sAk, const Operand &B, void *out, int epi,
                               const void *res, float *psum, float *psq, hipStream_t st)
{
    WaveConvArgs a;
    a.N = N;
    a.M = M;
    a.K = K;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    a.numTiles = (int)((a.Q + 127u) / 128u);
    a.divHW = make_div((uint32_t)HW);
    a.w = w;
    a.sAm = sAm;
    a.sAk = sAk;
    a.p0 = B.p0;
    a.p1 = B.p1;
    a.c0 = B.c0;
    a.c1 = B.c1;
    a.c2 = B.c2;
    a.gate = B.gate;
    a.out = out;
    a.res = res;
    a.psum = psum;
    a.psq = psq;
    const int grid = wave_conv_grid(kind, a.numTiles);
    a.NP = grid;
    return bf16 ? wave_dispatch<bf16_t>(a, kind, B.pro, epi, grid, st)
                : wave_dispatch<float>(a, kind, B.pro, epi, grid, st);
}

// ---- wgrad_cl ------------------------------------------------------------------------------------
// dW[a][b] = sum_{n,pix} U[n,a,pix] * V[n,b,pix], Ma <= 32*MTA (MTA <= 2, the narrow side),
// Mb <= 256 (one wavefront per 32 channels of the wide side).  Output element (a,b) is
// written at partial[split*Ma*Mb + a*sOa + b*sOb].

struct WgradClArgs {
    int N, Ma, Mb, HW;
    uint32_t Q;
    int numChunks, chunksPerWg; // 32-pixel chunks
    FastDiv divHW;
    const void *u0, *u1;
    const float *uc0, *uc1, *uc2, *ugate;
    const void *v0, *v1;
    const float *vc0, *vc1, *vc2, *vgate;
    int sOa, sOb;
    float *partial;
};

// Loads this lane's channel `c` of an operand for pixels [q, q+4) and applies its prologue.
template <typename T, int PRO>
__device__ __forceinline__ void load_chan4(const void *p0, const void *p1, const float *gate,
                                           int C, int HW, FastDiv divHW, uint32_t q, int c, float k0,
                                           float k1, float k2, float (&v)[4])
{
    const uint32_t n = fdiv(q, divHW);
    const size_t idx = ((size_t)n * C + c) * HW + (q - n * (uint32_t)HW);
    load4<T>((const T *)p0, idx, v);
    if (PRO == PRO_BNBWD) {
        float raw[4];
        load4<T>((const T *)p1, idx, raw);
#pragma unroll
        for (int r = 0; r < 4; ++r)
            v[r] = fmaf(k0, v[r], fmaf(k1, raw[r], k2));
    } else if (PRO == PRO_BNSWISH_GATE) {
        const float g = gate[(size_t)n * C + c];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            v[r] = swishf(fmaf(v[r], k0, k1)) * g;
    }
}

template <typename T, int MTA, int PROU, int PROV>
__global__ __launch_bounds__(512) void wgrad_cl_kernel(WgradClArgs a)
{
    const int lane = threadIdx.x & 63, t = threadIdx.x >> 6;
    const int h = lane >> 5, c = lane & 31;
    const int b = 32 * t + c;
    const bool bok = b < a.Mb;
    float vk0 = 0.f, vk1 = 0.f, vk2 = 0.f;
    if (bok && PROV != PRO_NONE) {
        vk0 = a.vc0[b];
        vk1 = a.vc1[b];
        if (PROV == PRO_BNBWD)
            vk2 = a.vc2[b];
    }
    float uk0[MTA], uk1[MTA], uk2[MTA];
    bool aok[MTA];
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta) {
        const int ai = 32 * ta + c;
        aok[ta] = ai < a.Ma;
        uk0[ta] = uk1[ta] = uk2[ta] = 0.f;
        if (aok[ta] && PROU != PRO_NONE) {
            uk0[ta] = a.uc0[ai];
            uk1[ta] = a.uc1[ai];
            if (PROU == PRO_BNBWD)
                uk2[ta] = a.uc2[ai];
        }
    }
    float16v acc[MTA];
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta)
        acc[ta] = (float16v){0};

    const int cBeg = blockIdx.x * a.chunksPerWg;
    const int cEnd = (cBeg + a.chunksPerWg < a.numChunks) ? cBeg + a.chunksPerWg : a.numChunks;
    for (int ch = cBeg; ch < cEnd; ++ch) {
        const uint32_t q0 = (uint32_t)ch * 32u;
        float vv[4][4], uu[MTA][4][4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const uint32_t q = q0 + 8 * jj + 4 * h;
            const bool qok = q < a.Q;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                vv[jj][r] = 0.f;
            if (qok && bok)
                load_chan4<T, PROV>(a.v0, a.v1, a.vgate, a.Mb, a.HW, a.divHW, q, b, vk0, vk1, vk2,
                                    vv[jj]);
#pragma unroll
            for (int ta = 0; ta < MTA; ++ta) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    uu[ta][jj][r] = 0.f;
                if (qok && aok[ta])
                    load_chan4<T, PROU>(a.u0, a.u1, a.ugate, a.Ma, a.HW, a.divHW, q, 32 * ta + c,
                                        uk0[ta], uk1[ta], uk2[ta], uu[ta][jj]);
            }
        }
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int ta = 0; ta < MTA; ++ta)
                    acc[ta] = __builtin_amdgcn_mfma_f32_32x32x2f32(uu[ta][jj][r], vv[jj][r], acc[ta],
                                                                   0, 0, 0);
    }
    float *dst = a.partial + (size_t)blockIdx.x * a.Ma * a.Mb;
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int ai = 32 * ta + 8 * (q >> 2) + 4 * h + (q & 3);
            if (ai < a.Ma && bok)
                dst[(size_t)ai * a.sOa + (size_t)b * a.sOb] = acc[ta][q];
        }
}

// Orientation and split count; returns false when the shape is not covered.
bool wgrad_cl_plan(int Ma, int Mb, int N, int HW, bool *swap, int *splits)
{
    if (HW % 4 != 0)
        return false;
    const int lo = Ma < Mb ? Ma : Mb, hi = Ma < Mb ? Mb : Ma;
    if (lo > 64 || hi > 256)
        return false;
    *swap = Ma > Mb; // the narrow side must be the U operand
    const long long chunks = ((long long)N * HW + 31) / 32;
    long long wg = chunks < 512 ? chunks : 512;
    const long long per = (chunks + wg - 1) / wg;
    *splits = (int)((chunks + per - 1) / per);
    return true;
}

template <typename T>
static hipError_t wgrad_cl_dispatch(const WgradClArgs &a, int mta, int pu, int pv, dim3 grid,
                                    dim3 block, hipStream_t st)
{
#define MBK_CASE(MTA, PU, PV)                                                                     \
    if (mta == MTA && pu == PU && pv == PV) {                                                     \
        hipLaunchKernelGGL((wgrad_cl_kernel<T, MTA, PU, PV>), grid, block, 0, st, a);             \
        return hipGetLastError();                                                                 \
    }
    MBK_CASE(1, PRO_BNBWD, PRO_NONE)
    MBK_CASE(1, PRO_BNBWD, PRO_BNSWISH_GATE)
    MBK_CASE(1, PRO_NONE, PRO_BNBWD)
    MBK_CASE(1, PRO_BNSWISH_GATE, PRO_BNBWD)
    MBK_CASE(2, PRO_BNBWD, PRO_NONE)
    MBK_CASE(2, PRO_BNBWD, PRO_BNSWISH_GATE)
    MBK_CASE(2, PRO_NONE, PRO_BNBWD)
    MBK_CASE(2, PRO_BNSWISH_GATE, PRO_BNBWD)
#undef MBK_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_wgrad_cl(bool bf16, int N, int Ma, int Mb, int HW, const Operand &U,
                           const Operand &V, float *partial, int *splits_out, hipStream_t st)
{
    bool swap;
    int splits;
    if (!wgrad_cl_plan(Ma, Mb, N, HW, &swap, &splits))
        return hipErrorInvalidValue;
    const Operand &u = swap ? V : U;
    const Operand &v = swap ? U : V;
    WgradClArgs a;
    a.N = N;
    a.Ma = swap ? Mb : Ma;
    a.Mb = swap ? Ma : Mb;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    a.numChunks = (int)((a.Q + 31u) / 32u);
    a.chunksPerWg = (a.numChunks + splits - 1) / splits;
    a.divHW = make_div((uint32_t)HW);
    a.u0 = u.p0;
    a.u1 = u.p1;
    a.uc0 = u.c0;
    a.uc1 = u.c1;
    a.uc2 = u.c2;
    a.ugate = u.gate;
    a.v0 = v.p0;
    a.v1 = v.p1;
    a.vc0 = v.c0;
    a.vc1 = v.c1;
    a.vc2 = v.c2;
    a.vgate = v.gate;
    // the caller's result is dW[Ma][Mb] row-major in its own orientation
    a.sOa = swap ? 1 : Mb;
    a.sOb = swap ? Mb : 1;
    a.partial = partial;
    *splits_out = splits;
    const int mta = (a.Ma + 31) / 32, mtb = (a.Mb + 31) / 32;
    dim3 grid((unsigned)splits), block((unsigned)(64 * mtb));
    return bf16 ? wgrad_cl_dispatch<bf16_t>(a, mta, u.pro, v.pro, grid, block, st)
                : wgrad_cl_dispatch<float>(a, mta, u.pro, v.pro, grid, block, st);
}

} // namespace mbk
