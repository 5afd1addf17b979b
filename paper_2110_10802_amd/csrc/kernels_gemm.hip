// 1x1 convolutions as N-batched GEMMs on the gfx950 matrix cores.
//
// A 1x1 convolution in NCHW is out_n[M x HW] = A[M x K] * B_n[K x HW] with no im2col
// copy (the paper lowers convolutions to matrix products, section "ONNX on SDFG").  The
// pixel axis is the contiguous one, so it is put on the MFMA column axis: every
// accumulator register then holds 32 consecutive pixels of one output channel across
// lanes 0..31 and stores are 128-byte runs.
//
// The B operand is produced by an elementwise prologue while it is staged into LDS
// (Swish(BN(.))*gate for the projection conv, the BN-backward expression for the two
// data-gradient convs), so those intermediates never exist in HBM (the paper's
// SubgraphFusion / TaskletFusion recompute knob, sections "Local Data Movement
// Reduction" and "Backpropagation and Data Movement").
#include "mbconv_dev.h"
#include "mbconv_launch.h"

namespace mbk {

typedef float float16v __attribute__((ext_vector_type(16)));

struct DevOperand {
    const void *p0, *p1;
    const float *c0, *c1, *c2, *gate;
};

template <typename T, int PRO>
__device__ __forceinline__ float load_operand(const DevOperand &o, int n, int c, int C, int HW,
                                              int pix)
{
    const size_t idx = ((size_t)n * C + c) * HW + pix;
    const float v = ld<T>((const T *)o.p0, idx);
    if (PRO == PRO_NONE) {
        return v;
    } else if (PRO == PRO_BNSWISH_GATE) {
        const float y = fmaf(v, o.c0[c], o.c1[c]);
        return actf(y) * o.gate[(size_t)n * C + c];
    } else {
        const float raw = ld<T>((const T *)o.p1, idx);
        return fmaf(o.c0[c], v, fmaf(o.c1[c], raw, o.c2[c]));
    }
}

struct Conv1x1Args {
    int N, M, K, HW;
    long long Q; // N*HW
    FastDiv divHW;
    const void *w;
    int sAm, sAk;
    DevOperand B;
    void *out;
    const void *res;
    float *psum, *psq;
    int NT;
    void *sc_store; // optional: receives the staged B operand (STORE policy), same layout as B
};

// Workgroup tile: 64 output channels x 128 pixels, K consumed 16 at a time.
// 4 waves as 2 (channels) x 2 (pixels); each wave owns a 32 x 64 block = two
// v_mfma_f32_32x32x2_f32 accumulators.
template <typename T, int PRO, int EPI>
__global__ __launch_bounds__(256) void conv1x1_kernel(Conv1x1Args a)
{
    constexpr int BM = 64, BQ = kConvBQ, BK = 16;
    __shared__ float As[BK][BM];
    __shared__ float Bs[BK][BQ];
    __shared__ float red[2][BM][2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wq = wave & 1;
    const int m0 = blockIdx.y * BM;
    const long long q0 = (long long)blockIdx.x * BQ;

    // B staging: this thread always stages pixel column bq, rows bk0, bk0+2, ...
    const int bq = tid & (BQ - 1), bk0 = tid >> 7;
    const long long qb = q0 + bq;
    const bool bvalid = qb < a.Q;
    int bn = 0, bpix = 0;
    if (bvalid) {
        bn = (int)fdiv((uint32_t)qb, a.divHW);
        bpix = (int)(qb - (long long)bn * a.HW);
    }

    float16v acc0 = {0}, acc1 = {0};
    for (int k0 = 0; k0 < a.K; k0 += BK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = tid + 256 * i;
            const int m = id & (BM - 1), kk = id >> 6;
            const int gm = m0 + m, gk = k0 + kk;
            float v = 0.f;
            if (gm < a.M && gk < a.K)
                v = ld<T>((const T *)a.w, (size_t)gm * a.sAm + (size_t)gk * a.sAk);
            As[kk][m] = v;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int kk = bk0 + 2 * i, gk = k0 + kk;
            float v = 0.f;
            if (bvalid && gk < a.K) {
                v = load_operand<T, PRO>(a.B, bn, gk, a.K, a.HW, bpix);
                if (PRO == PRO_BNSWISH_GATE && a.sc_store && blockIdx.y == 0)
                    st<T>((T *)a.sc_store, ((size_t)bn * a.K + gk) * a.HW + bpix, v);
            }
            Bs[kk][bq] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            const float av = As[kk + (lane >> 5)][wm * 32 + (lane & 31)];
            const float b0 = Bs[kk + (lane >> 5)][wq * 64 + (lane & 31)];
            const float b1 = Bs[kk + (lane >> 5)][wq * 64 + 32 + (lane & 31)];
            acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, b0, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, b1, acc1, 0, 0, 0);
        }
        __syncthreads();
    }

    // Accumulator register r of lane l is out[row 8*(r/4)+4*(l/32)+r%4][col l%32].
    float rs[16], rq[16];
#pragma unroll
    for (int r = 0; r < 16; ++r)
        rs[r] = rq[r] = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const long long q = q0 + wq * 64 + t * 32 + (lane & 31);
        const bool valid = q < a.Q;
        int n = 0, pix = 0;
        if (valid) {
            n = (int)fdiv((uint32_t)q, a.divHW);
            pix = (int)(q - (long long)n * a.HW);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            float v = t == 0 ? acc0[r] : acc1[r];
            if (valid && m < a.M) {
                const size_t idx = ((size_t)n * a.M + m) * a.HW + pix;
                if (EPI == EPI_RES)
                    v += ld<T>((const T *)a.res, idx);
                st<T>((T *)a.out, idx, v);
                if (EPI == EPI_STATS) {
                    const float sv = as_stored<T>(v);
                    rs[r] += sv;
                    rq[r] += sv * sv;
                }
            }
        }
    }
    if (EPI == EPI_STATS) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float s = half_wave_sum(rs[r]);
            const float s2 = half_wave_sum(rq[r]);
            if ((lane & 31) == 0) {
                const int row = wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                red[0][row][wq] = s;
                red[1][row][wq] = s2;
            }
        }
        __syncthreads();
        if (tid < BM && m0 + tid < a.M) {
            a.psum[(size_t)(m0 + tid) * a.NT + blockIdx.x] = red[0][tid][0] + red[0][tid][1];
            a.psq[(size_t)(m0 + tid) * a.NT + blockIdx.x] = red[1][tid][0] + red[1][tid][1];
        }
    }
}

static DevOperand to_dev(const Operand &o)
{
    DevOperand d;
    d.p0 = o.p0;
    d.p1 = o.p1;
    d.c0 = o.c0;
    d.c1 = o.c1;
    d.c2 = o.c2;
    d.gate = o.gate;
    return d;
}

template <typename T>
static hipError_t conv1x1_dispatch(const Conv1x1Args &a, int pro, int epi, dim3 grid, hipStream_t st)
{
#define MBK_CASE(P, E)                                                                            \
    if (pro == P && epi == E) {                                                                   \
        hipLaunchKernelGGL((conv1x1_kernel<T, P, E>), grid, dim3(256), 0, st, a);                 \
        return hipGetLastError();                                                                 \
    }
    MBK_CASE(PRO_NONE, EPI_STATS)
    MBK_CASE(PRO_BNSWISH_GATE, EPI_STATS)
    MBK_CASE(PRO_BNBWD, EPI_NONE)
    MBK_CASE(PRO_BNBWD, EPI_RES)
#undef MBK_CASE
    return hipErrorInvalidValue;
}

// kernels_wave.hip
int wave_conv_kind(int M, int K, int HW);
int wave_conv_num_partials(int kind, int N, int M, int HW);
hipError_t launch_wave_conv1x1(bool bf16, int kind, int N, int M, int K, int HW, const void *w,
                               int sAm, int sAk, const Operand &B, void *out, int epi,
                               const void *res, float *psum, float *psq, hipStream_t st);
bool wgrad_cl_plan(int Ma, int Mb, int N, int HW, bool *swap, int *splits);
hipError_t launch_wgrad_cl(bool bf16, int N, int Ma, int Mb, int HW, const Operand &U,
                           const Operand &V, float *partial, int *splits_out, hipStream_t st);

// kernels_big.hip
bool big_conv_plan(int N, int M, int K, int HW, int *wt, int *qtiles, int *splits);
size_t big_conv_splitk_floats(int N, int M, int K, int HW);
hipError_t launch_big_conv1x1(bool bf16, int N, int M, int K, int HW, const void *w, int sAm,
                              int sAk, const Operand &B, void *out, int epi, const void *res,
                              float *psum, float *psq, float *splitk_ws, hipStream_t st);
bool big_wgrad_plan(int Ma, int Mb, int N, int HW, int *wt, int *splits);
hipError_t launch_big_wgrad(bool bf16, int N, int Ma, int Mb, int HW, const Operand &U,
                            const Operand &V, float *partial, int *splits_out, hipStream_t st);

// kernels_bf.hip
bool bf_conv_plan(int N, int M, int K, int HW, int *qtiles, int *splits);
size_t bf_conv_splitk_floats(int N, int M, int K, int HW);
hipError_t launch_bf_conv1x1(int N, int M, int K, int HW, const void *w, int sAm, int sAk,
                             const Operand &B, void *out, int epi, const void *res, float *psum,
                             float *psq, float *splitk_ws, hipStream_t st);
bool bf_wgrad_plan(int Ma, int Mb, int N, int HW, int *splits);
hipError_t launch_bf_wgrad(int N, int Ma, int Mb, int HW, const Operand &U, const Operand &V,
                           float *partial, int *splits_out, hipStream_t st);

// kernels_x3.hip
bool x3_conv_plan(int N, int M, int K, int HW, int *qtiles, int *splits);
size_t x3_conv_splitk_floats(int N, int M, int K, int HW);
hipError_t launch_x3_conv1x1(int N, int M, int K, int HW, const void *wimg, const Operand &B,
                             void *out, int epi, const void *res, float *psum, float *psq,
                             float *splitk_ws, hipStream_t st);
bool x3_wgrad_plan(int Ma, int Mb, int N, int HW, int *splits);
hipError_t launch_x3_wgrad(int N, int Ma, int Mb, int HW, const Operand &U, const Operand &V,
                           float *partial, int *splits_out, hipStream_t st);
hipError_t launch_x3_wgrad_pair(int N, int MaA, int MbA, int HWA, const Operand &UA, const Operand &VA,
                                float *partialA, int *splitsA, int MaB, int MbB, int HWB,
                                const Operand &UB, const Operand &VB, float *partialB, int *splitsB,
                                hipStream_t st);
#ifndef MBK_X3PAIR
#define MBK_X3PAIR 1
#endif
// kernels_big.hip
hipError_t launch_big_wgrad_pair(bool bf16, int N, int MaA, int MbA, int HWA, const Operand &UA,
                                 const Operand &VA, float *partialA, int *splitsA, int MaB, int MbB,
                                 int HWB, const Operand &UB, const Operand &VB, float *partialB,
                                 int *splitsB, hipStream_t st);
bool xw_conv_plan(int N, int M, int K, int HW, int pro, int epi, int *nt);
hipError_t launch_xw_conv1x1(int N, int M, int K, int HW, const void *wimg, const Operand &B,
                             void *out, int epi, float *psum, float *psq, hipStream_t st);
#ifndef MBK_X3
#define MBK_X3 1
#endif
#ifndef MBK_XW
#define MBK_XW 1
#endif
#ifndef MBK_X3W
#define MBK_X3W 1
#endif

// short contraction, many rows, a role the kernel has: weights resident in LDS (conv_xw)
static bool xw_applies(bool bf16, int N, int M, int K, int HW, bool stores_operand, int pro, int epi,
                       int *nt)
{
    return MBK_XW && !bf16 && !stores_operand && pro >= 0 && epi >= 0 && !wave_conv_kind(M, K, HW) &&
           xw_conv_plan(N, M, K, HW, pro, epi, nt);
}

// fp32 convolutions of the wide blocks run on the bf16 matrix cores from a weight image
bool conv1x1_uses_weight_image(bool bf16, int N, int M, int K, int HW, bool stores_operand, int pro,
                               int epi)
{
    int qtiles, splits;
    if (xw_applies(bf16, N, M, K, HW, stores_operand, pro, epi, &qtiles))
        return true;
    return MBK_X3 && !bf16 && !stores_operand && !wave_conv_kind(M, K, HW) &&
           x3_conv_plan(N, M, K, HW, &qtiles, &splits);
}

int conv1x1_image_lane_order(bool bf16, int N, int M, int K, int HW, bool stores_operand, int pro,
                             int epi)
{
    int nt;
    return xw_applies(bf16, N, M, K, HW, stores_operand, pro, epi, &nt) ? 1 : 0;
}

// which matrix-core instruction family serves a launch (values of mbconv_engine in mbconv.h)
int conv1x1_engine(bool bf16, int N, int M, int K, int HW, bool stores_operand, int pro, int epi)
{
    if (conv1x1_uses_weight_image(bf16, N, M, K, HW, stores_operand, pro, epi))
        return 3;
    int qtiles, splits;
    if (bf16 && !stores_operand && !wave_conv_kind(M, K, HW) && bf_conv_plan(N, M, K, HW, &qtiles, &splits))
        return 2;
    return 1;
}
int wgrad1x1_engine(bool bf16, int Ma, int Mb, int N, int HW)
{
    bool swap;
    int splits;
    if (MBK_X3W && !bf16 && x3_wgrad_plan(Ma, Mb, N, HW, &splits))
        return 3;
    if (wgrad_cl_plan(Ma, Mb, N, HW, &swap, &splits))
        return 1;
    if (bf16 && bf_wgrad_plan(Ma, Mb, N, HW, &splits))
        return 2;
    return 1;
}

int conv1x1_num_partials(bool bf16, int N, int M, int K, int HW, bool stores_operand, int pro,
                         int epi)
{
    const int kind = stores_operand ? 0 : wave_conv_kind(M, K, HW);
    if (kind)
        return wave_conv_num_partials(kind, N, M, HW);
    int wt, qtiles, splits;
    if (xw_applies(bf16, N, M, K, HW, stores_operand, pro, epi, &qtiles))
        return qtiles;
    if (bf16 && !stores_operand && bf_conv_plan(N, M, K, HW, &qtiles, &splits))
        return qtiles;
    if (conv1x1_uses_weight_image(bf16, N, M, K, HW, stores_operand)) {
        x3_conv_plan(N, M, K, HW, &qtiles, &splits);
        return qtiles;
    }
    if (!stores_operand && big_conv_plan(N, M, K, HW, &wt, &qtiles, &splits))
        return qtiles;
    return conv1x1_num_qtiles(N, HW);
}

size_t conv1x1_splitk_floats(bool bf16, int N, int M, int K, int HW, bool stores_operand)
{
    if (stores_operand || wave_conv_kind(M, K, HW))
        return 0;
    int qtiles, splits;
    if (bf16 && bf_conv_plan(N, M, K, HW, &qtiles, &splits))
        return bf_conv_splitk_floats(N, M, K, HW);
    if (conv1x1_uses_weight_image(bf16, N, M, K, HW, stores_operand))
        return x3_conv_splitk_floats(N, M, K, HW);
    return big_conv_splitk_floats(N, M, K, HW);
}

hipError_t launch_conv1x1(bool bf16, int N, int M, int K, int HW, const void *w, int sAm, int sAk,
                          const Operand &B, void *out, int epi, const void *res, float *psum,
                          float *psq, void *sc_store, float *splitk_ws, hipStream_t st,
                          const void *wimg)
{
    {
        int nt;
        if (xw_applies(bf16, N, M, K, HW, sc_store != nullptr, B.pro, epi, &nt)) {
            if (!wimg)
                return hipErrorInvalidValue;
            return launch_xw_conv1x1(N, M, K, HW, wimg, B, out, epi, psum, psq, st);
        }
    }
    if (conv1x1_uses_weight_image(bf16, N, M, K, HW, sc_store != nullptr)) {
        if (!wimg)
            return hipErrorInvalidValue;
        return launch_x3_conv1x1(N, M, K, HW, wimg, B, out, epi, res, psum, psq, splitk_ws, st);
    }
    const int kind = sc_store ? 0 : wave_conv_kind(M, K, HW);
    if (kind)
        return launch_wave_conv1x1(bf16, kind, N, M, K, HW, w, sAm, sAk, B, out, epi, res, psum,
                                   psq, st);
    {
        int wt, qtiles, splits;
        if (bf16 && !sc_store && (sAm == 1 || sAk == 1) && bf_conv_plan(N, M, K, HW, &qtiles, &splits))
            return launch_bf_conv1x1(N, M, K, HW, w, sAm, sAk, B, out, epi, res, psum, psq, splitk_ws,
                                     st);
        if (!sc_store && (sAm == 1 || sAk == 1) &&
            big_conv_plan(N, M, K, HW, &wt, &qtiles, &splits))
            return launch_big_conv1x1(bf16, N, M, K, HW, w, sAm, sAk, B, out, epi, res, psum, psq,
                                      splitk_ws, st);
    }
    Conv1x1Args a;
    a.N = N;
    a.M = M;
    a.K = K;
    a.HW = HW;
    a.Q = (long long)N * HW;
    a.divHW = make_div((uint32_t)HW);
    a.w = w;
    a.sAm = sAm;
    a.sAk = sAk;
    a.B = to_dev(B);
    a.out = out;
    a.res = res;
    a.psum = psum;
    a.psq = psq;
    a.NT = conv1x1_num_qtiles(N, HW);
    a.sc_store = sc_store;
    dim3 grid((unsigned)a.NT, (unsigned)((M + 63) / 64));
    return bf16 ? conv1x1_dispatch<bf16_t>(a, B.pro, epi, grid, st)
                : conv1x1_dispatch<float>(a, B.pro, epi, grid, st);
}

hipError_t launch_conv1x1_affine(bool bf16, int N, int M, int K, int HW, const void *w, int sAm,
                                 int sAk, const Operand &B, void *out, const void *res,
                                 const float *scale, const float *shift, hipStream_t st,
                                 const void *wimg)
{
    if (B.pro != PRO_BNSWISH_GATE)
        return hipErrorNotSupported;
    float *sc = const_cast<float *>(scale), *sh = const_cast<float *>(shift); // read only
    if (wave_conv_kind(M, K, HW) == 2)
        return launch_wave_conv1x1(bf16, 2, N, M, K, HW, w, sAm, sAk, B, out, EPI_AFFINE, res, sc, sh,
                                   st);
    if (wave_conv_kind(M, K, HW) || (sAm != 1 && sAk != 1) || HW % 4 != 0)
        return hipErrorNotSupported;
    int wt, qtiles, splits;
    if (bf16 && bf_conv_plan(N, M, K, HW, &qtiles, &splits))
        return splits == 1 ? launch_bf_conv1x1(N, M, K, HW, w, sAm, sAk, B, out, EPI_AFFINE, res, sc,
                                               sh, nullptr, st)
                           : hipErrorNotSupported;
    if (conv1x1_uses_weight_image(bf16, N, M, K, HW, false)) {
        x3_conv_plan(N, M, K, HW, &qtiles, &splits);
        if (splits != 1 || !wimg)
            return hipErrorNotSupported;
        return launch_x3_conv1x1(N, M, K, HW, wimg, B, out, EPI_AFFINE, res, sc, sh, nullptr, st);
    }
    if (big_conv_plan(N, M, K, HW, &wt, &qtiles, &splits) && splits == 1)
        return launch_big_conv1x1(bf16, N, M, K, HW, w, sAm, sAk, B, out, EPI_AFFINE, res, sc, sh,
                                  nullptr, st);
    return hipErrorNotSupported;
}

// ---- weight gradient ------------------------------------------------------------------------
// dW[a,b] = sum_q U[a,q]*V[b,q]: the contraction runs over all N*HW pixels, so it is
// split across workgroups; every workgroup writes its own partial tile and a second
// kernel adds the partials in a fixed order (no atomics: the paper's map-fission step,
// section "Guided Optimization Case Study: EfficientNet").

struct WgradArgs {
    int N, Ma, Mb, HW;
    long long Q, chunk;
    FastDiv divHW;
    DevOperand U, V;
    float *partial;
};

template <typename T, int PROU, int PROV>
__global__ __launch_bounds__(256) void wgrad1x1_kernel(WgradArgs a)
{
    constexpr int BA = 64, BB = 64, BQ = 32;
    __shared__ float Us[BQ][BA + 1];
    __shared__ float Vs[BQ][BB + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wa = wave >> 1, wb = wave & 1;
    const int a0 = blockIdx.x * BA, b0 = blockIdx.y * BB;
    const long long qbeg = (long long)blockIdx.z * a.chunk;
    const long long qend = (qbeg + a.chunk < a.Q) ? qbeg + a.chunk : a.Q;
    const int sq = tid & 31, r0 = tid >> 5;

    float16v acc = {0};
    for (long long qb = qbeg; qb < qend; qb += BQ) {
        const long long q = qb + sq;
        const bool valid = q < qend;
        int n = 0, pix = 0;
        if (valid) {
            n = (int)fdiv((uint32_t)q, a.divHW);
            pix = (int)(q - (long long)n * a.HW);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = r0 + 8 * i;
            float u = 0.f, v = 0.f;
            if (valid && a0 + r < a.Ma)
                u = load_operand<T, PROU>(a.U, n, a0 + r, a.Ma, a.HW, pix);
            if (valid && b0 + r < a.Mb)
                v = load_operand<T, PROV>(a.V, n, b0 + r, a.Mb, a.HW, pix);
            Us[sq][r] = u;
            Vs[sq][r] = v;
        }
        __syncthreads();
#pragma unroll
        for (int qq = 0; qq < BQ; qq += 2) {
            const float u = Us[qq + (lane >> 5)][wa * 32 + (lane & 31)];
            const float v = Vs[qq + (lane >> 5)][wb * 32 + (lane & 31)];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(u, v, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    float *dst = a.partial + (size_t)blockIdx.z * a.Ma * a.Mb;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int ai = a0 + wa * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const int bi = b0 + wb * 32 + (lane & 31);
        if (ai < a.Ma && bi < a.Mb)
            dst[(size_t)ai * a.Mb + bi] = acc[r];
    }
}

static long long wgrad_chunk(int Ma, int Mb, long long Q)
{
    const long long tiles = (long long)((Ma + 63) / 64) * ((Mb + 63) / 64);
    long long want = 512 / tiles; // workgroups along the contraction
    if (want < 1)
        want = 1;
    long long chunk = (Q + want - 1) / want;
    chunk = ((chunk + 31) / 32) * 32;
    if (chunk < 128)
        chunk = 128;
    return chunk;
}

int wgrad_splits(bool bf16, int Ma, int Mb, int N, int HW)
{
    bool swap;
    int splits;
    if (MBK_X3W && !bf16 && x3_wgrad_plan(Ma, Mb, N, HW, &splits))
        return splits;
    if (wgrad_cl_plan(Ma, Mb, N, HW, &swap, &splits))
        return splits;
    if (bf16 && bf_wgrad_plan(Ma, Mb, N, HW, &splits))
        return splits;
    int wt;
    if (big_wgrad_plan(Ma, Mb, N, HW, &wt, &splits))
        return splits;
    const long long Q = (long long)N * HW;
    const long long chunk = wgrad_chunk(Ma, Mb, Q);
    return (int)((Q + chunk - 1) / chunk);
}

// Second stage of a split reduction: out[i] = sum_k in[k*count+i].  A workgroup owns E*V
// consecutive outputs (V = 4 when count is a multiple of four: 16-byte loads); its G = 1024/E
// thread groups each add every G-th partial in ascending order (four independent running sums
// per thread to keep loads in flight), then the groups are combined by a fixed-shape tree in
// LDS.  No atomics, bitwise repeatable.
template <int V, int E>
__device__ __forceinline__ void reduce_splits_body(const float *__restrict__ in, int S, size_t count,
                                                   float *__restrict__ out, unsigned block)
{
    constexpr int G = 1024 / E; // thread groups of E lanes; the workgroup owns E*V outputs
    __shared__ float part[G][E * V + 1];
    const int e = threadIdx.x % E, grp = threadIdx.x / E;
    const size_t i = ((size_t)block * E + e) * V;
    float s[4][V];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < V; ++v)
            s[u][v] = 0.f;
    auto add = [&](int u, int k) __attribute__((always_inline)) {
        const float *p = in + (size_t)k * count + i;
        if (V == 4) {
            const float4 t = *reinterpret_cast<const float4 *>(p);
            s[u][0] += t.x;
            s[u][V > 1 ? 1 : 0] += t.y;
            s[u][V > 2 ? 2 : 0] += t.z;
            s[u][V > 3 ? 3 : 0] += t.w;
        } else {
            s[u][0] += p[0];
        }
    };
    if (i < count) {
        int k = grp;
        for (; k + 3 * G < S; k += 4 * G) {
            add(0, k);
            add(1, k + G);
            add(2, k + 2 * G);
            add(3, k + 3 * G);
        }
        for (; k < S; k += G)
            add(0, k);
    }
#pragma unroll
    for (int v = 0; v < V; ++v)
        part[grp][e * V + v] = (s[0][v] + s[1][v]) + (s[2][v] + s[3][v]);
    __syncthreads();
    for (int half = G / 2; half > 0; half >>= 1) {
        if (grp < half) {
#pragma unroll
            for (int v = 0; v < V; ++v)
                part[grp][e * V + v] += part[grp + half][e * V + v];
        }
        __syncthreads();
    }
    if (grp == 0 && i < count) {
#pragma unroll
        for (int v = 0; v < V; ++v)
            out[i + v] = part[0][e * V + v];
    }
}

// Up to two independent reductions in one launch (the workgroups of the second follow those of
// the first): two launches cost a launch latency more than the reductions themselves take.
// 16 lanes x 4 outputs per thread group with 16-byte loads (64 groups share the partial rows: a
// 144x24 gradient with 448 splits then runs on 108 workgroups, measured 0.8 us faster than 32
// lanes x 32 groups on 54), 32 lanes x 1 otherwise.
template <int V, int E>
__global__ __launch_bounds__(1024) void reduce_splits_kernel(SplitReduce a, SplitReduce b,
                                                             unsigned blocks_a)
{
    if (blockIdx.x < blocks_a)
        reduce_splits_body<V, E>(a.in, a.S, a.count, a.out, blockIdx.x);
    else
        reduce_splits_body<V, E>(b.in, b.S, b.count, b.out, blockIdx.x - blocks_a);
}

hipError_t launch_reduce_splits2(const SplitReduce &a, const SplitReduce &b, hipStream_t st)
{
    const auto wide = [](const SplitReduce &r) {
        return r.count % 4 == 0 && (((uintptr_t)r.in | (uintptr_t)r.out) & 15u) == 0;
    };
    const bool two = b.count > 0;
    if (wide(a) && (!two || wide(b))) {
        // lanes per thread group by the number of partial rows: a group adds every (1024/E)-th row,
        // so few rows want few, wide groups (with 64 groups and 16 rows three quarters of the
        // threads would idle)
        const int S = two ? (a.S < b.S ? a.S : b.S) : a.S;
#define MBK_GO(E)                                                                                 \
    {                                                                                             \
        const unsigned ba = (unsigned)((a.count / 4 + (E)-1) / (E));                              \
        const unsigned bb = two ? (unsigned)((b.count / 4 + (E)-1) / (E)) : 0u;                   \
        hipLaunchKernelGGL((reduce_splits_kernel<4, E>), dim3(ba + bb), dim3(1024), 0, st, a, b,  \
                           ba);                                                                   \
    }
        if (S >= 128)
            MBK_GO(16)
        else if (S >= 32)
            MBK_GO(32)
        else
            MBK_GO(64)
#undef MBK_GO
    } else {
        const unsigned ba = (unsigned)((a.count + 31) / 32);
        const unsigned bb = two ? (unsigned)((b.count + 31) / 32) : 0u;
        hipLaunchKernelGGL((reduce_splits_kernel<1, 32>), dim3(ba + bb), dim3(1024), 0, st, a, b, ba);
    }
    return hipGetLastError();
}

hipError_t launch_reduce_splits(const float *in, int S, size_t count, float *out, hipStream_t st)
{
    return launch_reduce_splits2({in, S, count, out}, {nullptr, 0, 0, nullptr}, st);
}

template <typename T>
static hipError_t wgrad_dispatch(const WgradArgs &a, int pu, int pv, dim3 grid, hipStream_t st)
{
#define MBK_CASE(PU, PV)                                                                          \
    if (pu == PU && pv == PV) {                                                                   \
        hipLaunchKernelGGL((wgrad1x1_kernel<T, PU, PV>), grid, dim3(256), 0, st, a);              \
        return hipGetLastError();                                                                 \
    }
    MBK_CASE(PRO_BNBWD, PRO_NONE)
    MBK_CASE(PRO_BNBWD, PRO_BNSWISH_GATE)
#undef MBK_CASE
    return hipErrorInvalidValue;
}

// Two weight gradients of one block (A and B, each as launch_wgrad1x1 takes it) in one launch
// where both are shapes of the split-operand kernel; the sums over their splits are described in
// *ra and *rb for the caller to launch.  hipErrorNotSupported (nothing was launched) unless
// wgrad1x1_pair_supported holds.
// 1: both are shapes of the split-operand kernel; 2: both go to the 64 x 64-tile kernel of
// kernels_big.hip with planes that are not a multiple of four pixels (the 7x7 stages); 0: no pair
static int wgrad1x1_pair_kind(bool bf16, int N, int MaA, int MbA, int HWA, int MaB, int MbB, int HWB)
{
    if (!MBK_X3PAIR)
        return 0;
    int s, wt;
    bool swap;
    const bool xa = MBK_X3W && !bf16 && x3_wgrad_plan(MaA, MbA, N, HWA, &s);
    const bool xb = MBK_X3W && !bf16 && x3_wgrad_plan(MaB, MbB, N, HWB, &s);
    if (xa && xb)
        return 1;
    const auto big = [&](bool x3, int Ma, int Mb, int HW) {
        return !x3 && HW % 4 != 0 && !wgrad_cl_plan(Ma, Mb, N, HW, &swap, &s) &&
               !(bf16 && bf_wgrad_plan(Ma, Mb, N, HW, &s)) && big_wgrad_plan(Ma, Mb, N, HW, &wt, &s) && wt == 5;
    };
    return big(xa, MaA, MbA, HWA) && big(xb, MaB, MbB, HWB) ? 2 : 0;
}
bool wgrad1x1_pair_supported(bool bf16, int N, int MaA, int MbA, int HWA, int MaB, int MbB, int HWB)
{
    return wgrad1x1_pair_kind(bf16, N, MaA, MbA, HWA, MaB, MbB, HWB) != 0;
}
hipError_t launch_wgrad1x1_pair(bool bf16, int N, int MaA, int MbA, int HWA, const Operand &UA,
                                const Operand &VA, float *partialA, float *dWA, SplitReduce *ra,
                                int MaB, int MbB, int HWB, const Operand &UB, const Operand &VB,
                                float *partialB, float *dWB, SplitReduce *rb, hipStream_t st)
{
    const int kind = wgrad1x1_pair_kind(bf16, N, MaA, MbA, HWA, MaB, MbB, HWB);
    if (!kind)
        return hipErrorNotSupported;
    int sa = 0, sb = 0;
    hipError_t e;
    if (kind == 1) {
        e = launch_x3_wgrad_pair(N, MaA, MbA, HWA, UA, VA, partialA, &sa, MaB, MbB, HWB, UB, VB, partialB, &sb,
                                 st);
        if (e == hipErrorNotSupported) {
            // a pair of kernel forms the launch does not have (e.g. a stored activation on the
            // projection side): one after the other
            e = launch_x3_wgrad(N, MaA, MbA, HWA, UA, VA, partialA, &sa, st);
            if (e == hipSuccess)
                e = launch_x3_wgrad(N, MaB, MbB, HWB, UB, VB, partialB, &sb, st);
        }
    } else {
        e = launch_big_wgrad_pair(bf16, N, MaA, MbA, HWA, UA, VA, partialA, &sa, MaB, MbB, HWB, UB, VB,
                                  partialB, &sb, st);
        if (e == hipErrorNotSupported) {
            e = launch_big_wgrad(bf16, N, MaA, MbA, HWA, UA, VA, partialA, &sa, st);
            if (e == hipSuccess)
                e = launch_big_wgrad(bf16, N, MaB, MbB, HWB, UB, VB, partialB, &sb, st);
        }
    }
    if (e != hipSuccess)
        return e;
    *ra = {partialA, sa, (size_t)MaA * MbA, dWA};
    *rb = {partialB, sb, (size_t)MaB * MbB, dWB};
    return hipSuccess;
}

hipError_t launch_wgrad1x1(bool bf16, int N, int Ma, int Mb, int HW, const Operand &U,
                           const Operand &V, float *partial, float *dW, SplitReduce *defer,
                           hipStream_t st)
{
    // second stage: launched here, or handed back for the caller to launch with another one
    const auto finish = [&](int splits) {
        const SplitReduce r = {partial, splits, (size_t)Ma * Mb, dW};
        if (defer) {
            *defer = r;
            return hipSuccess;
        }
        return launch_reduce_splits2(r, {nullptr, 0, 0, nullptr}, st);
    };
    {
        bool swap;
        int splits;
        if (MBK_X3W && !bf16 && x3_wgrad_plan(Ma, Mb, N, HW, &splits)) {
            hipError_t e = launch_x3_wgrad(N, Ma, Mb, HW, U, V, partial, &splits, st);
            if (e != hipSuccess)
                return e;
            return finish(splits);
        }
        if (wgrad_cl_plan(Ma, Mb, N, HW, &swap, &splits)) {
            hipError_t e = launch_wgrad_cl(bf16, N, Ma, Mb, HW, U, V, partial, &splits, st);
            if (e != hipSuccess)
                return e;
            return finish(splits);
        }
        if (bf16 && bf_wgrad_plan(Ma, Mb, N, HW, &splits)) {
            hipError_t e = launch_bf_wgrad(N, Ma, Mb, HW, U, V, partial, &splits, st);
            if (e != hipSuccess)
                return e;
            return finish(splits);
        }
        int wt;
        if (big_wgrad_plan(Ma, Mb, N, HW, &wt, &splits)) {
            hipError_t e = launch_big_wgrad(bf16, N, Ma, Mb, HW, U, V, partial, &splits, st);
            if (e != hipSuccess)
                return e;
            return finish(splits);
        }
    }
    WgradArgs a;
    a.N = N;
    a.Ma = Ma;
    a.Mb = Mb;
    a.HW = HW;
    a.Q = (long long)N * HW;
    a.chunk = wgrad_chunk(Ma, Mb, a.Q);
    a.divHW = make_div((uint32_t)HW);
    a.U = to_dev(U);
    a.V = to_dev(V);
    a.partial = partial;
    const int S = (int)((a.Q + a.chunk - 1) / a.chunk);
    dim3 grid((unsigned)((Ma + 63) / 64), (unsigned)((Mb + 63) / 64), (unsigned)S);
    hipError_t err = bf16 ? wgrad_dispatch<bf16_t>(a, U.pro, V.pro, grid, st)
                          : wgrad_dispatch<float>(a, U.pro, V.pro, grid, st);
    if (err != hipSuccess)
        return err;
    return finish(S);
}

} // namespace mbk
