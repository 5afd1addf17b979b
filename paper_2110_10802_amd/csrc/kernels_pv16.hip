// Register-direct 1x1 convolutions for the HBM-bound ("skinny") shapes, built on
// v_mfma_f32_16x16x4_f32 with four-pixel vectors.
//
// What decides the speed of a 24 <-> 144 channel 1x1 convolution on this chip is not flops but
// (a) 16-byte-per-lane global accesses (a dword-per-lane stream reaches under half the
// bandwidth) and (b) enough independent wavefronts: a batch-32 56x56 layer has only 100 k
// pixels, so tiles must be small.  Hence:
//
//   out[ch][pix] = sum_k W[ch][k] * act[k][pix],   C[i][j] += sum_k A[i][k] * B[k][j] with
//   A = weights     lane l holds A[i = l%16][k = l/16]          (i = output channel)
//   B = activations lane l holds B[k = l/16][j = l%16]          (j = group of 4 pixels)
//   C               lane l, register v holds C[i = 4*(l/16)+v][j = l%16]
//
// A lane loads FOUR consecutive pixels of one input channel (float4; one load instruction
// covers 4 input channels x 64 pixels, 256 contiguous bytes per channel) and feeds element r of
// the vector to MFMA number r, so accumulator C_r holds pixels 4j+r.  Register v of C_0..C_3
// is then four consecutive pixels of one output channel: stores are float4 too.  A tile is 64
// pixels; activations never pass through LDS; there is no barrier in a main loop.
//
//   conv_pe ("expand-like", few input channels, K <= 40): the activation tile (K/4 float4 per
//     lane) stays in registers; each wavefront of the workgroup produces 48 output channels.
//   conv_pr ("reduce-like", at most 32 output channels): the input channels are split over the
//     four wavefronts (each matrix core gets a quarter of the MFMAs); each wavefront then
//     finishes a quarter of the output channels after one exchange of partial tiles via LDS.
//
// The elementwise prologues (Swish(BN(.))*gate, BN backward) run on the activation registers
// between load and MFMA, so those tensors never exist in memory (recomputation instead of
// load/store: section "Backpropagation and Data Movement" of the paper).  Per-channel BN
// partial sums are reduced over the 16 lanes of a row with DPP row rotations (the paper's
// warp-collective reductions, section "Hardware Specialization").
#include "mbconv_dev.h"
#include "mbconv_launch.h"

namespace mbk {

typedef float float4v __attribute__((ext_vector_type(4)));

struct PvArgs {
    int N, M, K, HW;
    uint32_t Q; // N*HW, a multiple of 4
    int numTiles; // 64-pixel tiles
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
__device__ __forceinline__ void pv_load4(const T *p, size_t i, float (&v)[4]);
template <>
__device__ __forceinline__ void pv_load4<float>(const float *p, size_t i, float (&v)[4])
{
    const float4v t = *reinterpret_cast<const float4v *>(p + i);
    v[0] = t.x;
    v[1] = t.y;
    v[2] = t.z;
    v[3] = t.w;
}
template <>
__device__ __forceinline__ void pv_load4<bf16_t>(const bf16_t *p, size_t i, float (&v)[4])
{
    const uint2 t = *reinterpret_cast<const uint2 *>(&p[i]);
    v[0] = bf16_bits_to_float(t.x & 0xffffu);
    v[1] = bf16_bits_to_float(t.x >> 16);
    v[2] = bf16_bits_to_float(t.y & 0xffffu);
    v[3] = bf16_bits_to_float(t.y >> 16);
}
template <typename T>
__device__ __forceinline__ void pv_store4(T *p, size_t i, const float (&v)[4]);
template <>
__device__ __forceinline__ void pv_store4<float>(float *p, size_t i, const float (&v)[4])
{
    float4v t = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<float4v *>(p + i) = t;
}
template <>
__device__ __forceinline__ void pv_store4<bf16_t>(bf16_t *p, size_t i, const float (&v)[4])
{
    uint2 t;
    t.x = bf16_pack2(v[0], v[1]);
    t.y = bf16_pack2(v[2], v[3]);
    *reinterpret_cast<uint2 *>(&p[i]) = t;
}

// One float4 of activations of input channel k, image n, in two steps: the raw loads, and the
// prologue (PRO_* in the header) applied to them.  The kernels issue the raw loads of a whole
// batch first and fence the instruction scheduler before the arithmetic: left alone, the
// compiler sinks every load next to its use to save registers, which serialises the batch into
// one memory round trip per load.
template <int PRO>
struct PvRaw {
    float v[4];
    float r[PRO == PRO_BNBWD ? 4 : 1];
    float g;
};
template <typename T, int PRO>
__device__ __forceinline__ void pv_load_raw(const PvArgs &a, size_t idx, uint32_t n, int k, PvRaw<PRO> &o)
{
    pv_load4<T>((const T *)a.p0, idx, o.v);
    if constexpr (PRO == PRO_BNBWD)
        pv_load4<T>((const T *)a.p1, idx, o.r);
    if (PRO == PRO_BNSWISH_GATE)
        o.g = a.gate[(size_t)n * a.K + k];
}
template <int PRO>
__device__ __forceinline__ void pv_apply(const PvRaw<PRO> &o, int k, const float *coef, int cstride,
                                         float (&v)[4])
{
    if (PRO == PRO_BNBWD) {
        const float c0 = coef[k], c1 = coef[cstride + k], c2 = coef[2 * cstride + k];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            v[r] = fmaf(c0, o.v[r], fmaf(c1, o.r[PRO == PRO_BNBWD ? r : 0], c2));
    } else if (PRO == PRO_BNSWISH_GATE) {
        const float sc = coef[k], sh = coef[cstride + k];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            v[r] = actf(fmaf(o.v[r], sc, sh)) * o.g;
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            v[r] = o.v[r];
    }
}

template <int PRO>
__device__ __forceinline__ void pv_stage_coef(const PvArgs &a, float *coef, int cstride)
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
    __syncthreads();
}

// ---- conv_pe: few input channels --------------------------------------------------------------
constexpr int kPeTT = 3;      // 16-channel tiles per wavefront (48 output channels)
constexpr int kPeMaxWaves = 8; // M <= 384

template <typename T, int KS4, int PRO, int EPI>
__global__ __launch_bounds__(64 * kPeMaxWaves) void conv_pe_kernel(PvArgs a)
{
    __shared__ float coef[3 * 4 * KS4];
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform
    const int kk = lane >> 4, j = lane & 15;
    pv_stage_coef<PRO>(a, coef, 4 * KS4);

    // this wavefront's weights in A-operand order: wreg[t][s] = W(ch = 16*(wv*TT+t) + l%16, k = 4s + l/16)
    float wreg[kPeTT][KS4];
#pragma unroll
    for (int t = 0; t < kPeTT; ++t)
#pragma unroll
        for (int s = 0; s < KS4; ++s) {
            const int m = 16 * (wv * kPeTT + t) + j, k = 4 * s + kk;
            wreg[t][s] = (m < a.M && k < a.K)
                             ? ld<T>((const T *)a.w, (size_t)m * a.sAm + (size_t)k * a.sAk)
                             : 0.f;
        }

    float ssum[kPeTT][4], ssq[kPeTT][4];
#pragma unroll
    for (int t = 0; t < kPeTT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            ssum[t][v] = ssq[t][v] = 0.f;

    for (int tile = blockIdx.x; tile < a.numTiles; tile += gridDim.x) {
        const uint32_t qv = (uint32_t)tile * 64u + 4u * j;
        const bool valid = qv < a.Q;
        const uint32_t n = valid ? fdiv(qv, a.divHW) : 0;
        const uint32_t pix = valid ? qv - n * (uint32_t)a.HW : 0;
        PvRaw<PRO> raw[KS4];
#pragma unroll
        for (int s = 0; s < KS4; ++s) {
            const int k = min(4 * s + kk, a.K - 1); // past the end: a valid address, masked below
            pv_load_raw<T, PRO>(a, ((size_t)n * a.K + k) * a.HW + pix, n, k, raw[s]);
        }
        __builtin_amdgcn_sched_barrier(0);
        float bv[KS4][4];
#pragma unroll
        for (int s = 0; s < KS4; ++s) {
            const int k = 4 * s + kk;
            pv_apply<PRO>(raw[s], min(k, a.K - 1), coef, 4 * KS4, bv[s]);
            if (!(valid && k < a.K)) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    bv[s][r] = 0.f;
            }
        }
#pragma unroll
        for (int t = 0; t < kPeTT; ++t) {
            float4v acc[4];
#pragma unroll
            for (int r = 0; r < 4; ++r)
                acc[r] = (float4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KS4; ++s)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[r] = __builtin_amdgcn_mfma_f32_16x16x4f32(wreg[t][s], bv[s][r], acc[r], 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = 16 * (wv * kPeTT + t) + 4 * kk + v;
                if (valid && m < a.M) {
                    const size_t idx = ((size_t)n * a.M + m) * a.HW + pix;
                    float o[4] = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
                    if (EPI == EPI_RES) {
                        float rr[4];
                        pv_load4<T>((const T *)a.res, idx, rr);
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            o[r] += rr[r];
                    }
                    pv_store4<T>((T *)a.out, idx, o);
                    if (EPI == EPI_STATS) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const float sv = as_stored<T>(o[r]);
                            ssum[t][v] += sv;
                            ssq[t][v] = fmaf(sv, sv, ssq[t][v]);
                        }
                    }
                }
            }
        }
    }
    if (EPI == EPI_STATS) {
#pragma unroll
        for (int t = 0; t < kPeTT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float s = row16_sum(ssum[t][v]);
                const float s2 = row16_sum(ssq[t][v]);
                const int m = 16 * (wv * kPeTT + t) + 4 * kk + v;
                if (j == 0 && m < a.M) {
                    a.psum[(size_t)m * a.NP + blockIdx.x] = s;
                    a.psq[(size_t)m * a.NP + blockIdx.x] = s2;
                }
            }
    }
}

// ---- conv_pr: at most 32 output channels --------------------------------------------------------
// Wavefront w contracts the input-channel quads [w*KSW, (w+1)*KSW) of the tile into two
// 16-channel accumulator tiles; then output-channel registers (t, v) with 2*t + v/2 == g go to
// wavefront g, which adds the four partials in wavefront order and stores channels
// 16*(g/2) + 4*(l/16) + 2*(g%2) + {0,1}.
// The share of every wavefront is padded to KSWp quads (a multiple of the batch size U); padded
// quads have zero weights in LDS and read a clamped, valid address, so the load / MFMA loops
// carry no bounds checks.
template <typename T, int PRO, int EPI, int U>
__global__ __launch_bounds__(256) void conv_pr_kernel(PvArgs a, int KSWp)
{
    extern __shared__ float lds[];
    const int KS4p = 4 * KSWp;
    float *coef = lds;                 // [3][4*KS4p]
    float *xch = lds + 12 * KS4p;      // [4 src][4 dst][8 values][64 lanes]
    float *wl = xch + 16 * 8 * 64;     // [KS4p][2][64]: weights in A-operand order
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform, keep it scalar
    const int kk = lane >> 4, j = lane & 15;
    // wl[(s*2+t)*64 + l] = W(ch = 16t + l%16, k = 4s + l/16), zero outside M x K
    // (KS4p*128 entries, 256 threads: KS4p/2 = 2*KSWp per thread, six loads in flight at a time:
    // a load-store loop would pay one memory round trip per entry)
    for (int i0 = 0; i0 < 2 * KSWp; i0 += 6) {
        float wv[6];
#pragma unroll
        for (int u = 0; u < 6; ++u) {
            const int idx = (int)threadIdx.x + 256 * (i0 + u);
            const int ln = idx & 63, st_ = idx >> 6;
            const int m = 16 * (st_ & 1) + (ln & 15), k = 4 * (st_ >> 1) + (ln >> 4);
            const bool ok = i0 + u < 2 * KSWp && m < a.M && k < a.K;
            wv[u] = and_mask(ld<T>((const T *)a.w, ok ? (size_t)m * a.sAm + (size_t)k * a.sAk : 0),
                             ok ? 0xffffffffu : 0u);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 6; ++u)
            if (i0 + u < 2 * KSWp)
                wl[(int)threadIdx.x + 256 * (i0 + u)] = wv[u];
    }
    if (PRO == PRO_NONE)
        __syncthreads();
    pv_stage_coef<PRO>(a, coef, 4 * KS4p); // ends with a barrier when there is a prologue

    float ssum[2] = {0.f, 0.f}, ssq[2] = {0.f, 0.f};
    const int sBeg = w * KSWp;
    const int tOwn = w >> 1, vOwn = 2 * (w & 1);
    const int kLast = a.K - 1;

    // geometry of this lane's four pixels in a tile
    struct Geo {
        bool valid;
        uint32_t n, pix;
        size_t base;
    };
    auto geo_of = [&](int tile) __attribute__((always_inline)) {
        Geo g;
        const uint32_t qv = (uint32_t)tile * 64u + 4u * j;
        g.valid = tile < a.numTiles && qv < a.Q;
        const uint32_t qs = g.valid ? qv : 0u; // lanes past the end read pixel 0 and store nothing
        g.n = fdiv(qs, a.divHW);
        g.pix = qs - g.n * (uint32_t)a.HW;
        g.base = (size_t)g.n * a.K * a.HW + g.pix;
        return g;
    };
    auto load_batch = [&](const Geo &g, int u0, PvRaw<PRO>(&raw)[U]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int k = 4 * (sBeg + u0 + u) + kk;
            k = k < kLast ? k : kLast;
            pv_load_raw<T, PRO>(a, g.base + (size_t)k * a.HW, g.n, k, raw[u]);
        }
    };
    auto compute_batch = [&](int u0, const PvRaw<PRO>(&raw)[U], float4v(&acc)[2][4]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = sBeg + u0 + u;
            int k = 4 * s + kk;
            k = k < kLast ? k : kLast;
            float bv[4];
            pv_apply<PRO>(raw[u], k, coef, 4 * KS4p, bv);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const float wv = wl[(s * 2 + t) * 64 + lane];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[t][r] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv, bv[r], acc[t][r], 0, 0, 0);
            }
        }
    };
    // residual rows this wavefront finishes (EPI_RES), loaded together with the tile's batch
    auto load_res = [&](const Geo &g, float(&rr)[2][4]) __attribute__((always_inline)) {
#pragma unroll
        for (int dv = 0; dv < 2; ++dv) {
            int m = 16 * tOwn + 4 * kk + vOwn + dv;
            m = m < a.M ? m : a.M - 1;
            pv_load4<T>((const T *)a.res, ((size_t)g.n * a.M + m) * a.HW + g.pix, rr[dv]);
        }
    };
    // exchange partial tiles: every wavefront publishes, per destination g, the two accumulator
    // registers that g finishes (tile g/2, registers 2*(g%2) + {0,1}); then finish, store, stats
    auto finish_tile = [&](const Geo &g, const float4v(&acc)[2][4], const float(&rr)[2][4]) __attribute__((always_inline)) {
        __syncthreads(); // the previous tile's buffer has been consumed
#pragma unroll
        for (int gd = 0; gd < 4; ++gd)
#pragma unroll
            for (int dv = 0; dv < 2; ++dv)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    xch[(((w * 4 + gd) * 8) + dv * 4 + r) * 64 + lane] = acc[gd >> 1][r][2 * (gd & 1) + dv];
        __syncthreads();
#pragma unroll
        for (int dv = 0; dv < 2; ++dv) {
            float o[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float sacc = 0.f;
#pragma unroll
                for (int src = 0; src < 4; ++src)
                    sacc += xch[(((src * 4 + w) * 8) + dv * 4 + r) * 64 + lane];
                o[r] = sacc;
            }
            const int m = 16 * tOwn + 4 * kk + vOwn + dv;
            if (g.valid && m < a.M) {
                const size_t idx = ((size_t)g.n * a.M + m) * a.HW + g.pix;
                if (EPI == EPI_RES) {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        o[r] += rr[dv][r];
                }
                if (EPI == EPI_AFFINE) { // psum / psq carry the row's scale and shift
                    const float osc = a.psum[m], osh = a.psq[m];
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        o[r] = fmaf(o[r], osc, osh) + (a.res ? rr[dv][r] : 0.f);
                }
                pv_store4<T>((T *)a.out, idx, o);
                if (EPI == EPI_STATS) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float sv = as_stored<T>(o[r]);
                        ssum[dv] += sv;
                        ssq[dv] = fmaf(sv, sv, ssq[dv]);
                    }
                }
            }
        }
    };

    if (KSWp == U) {
        // One batch per tile: the next tile's loads are issued right after this tile's MFMAs,
        // so they are in flight during the exchange, the stores and the two barriers.
        PvRaw<PRO> raw[U];
        float rnext[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        Geo g = geo_of(blockIdx.x);
        if ((int)blockIdx.x < a.numTiles) {
            load_batch(g, 0, raw);
            if (EPI == EPI_RES || (EPI == EPI_AFFINE && a.res))
                load_res(g, rnext);
        }
        for (int tile = blockIdx.x; tile < a.numTiles; tile += gridDim.x) {
            __builtin_amdgcn_sched_barrier(0);
            float4v acc[2][4];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[t][r] = (float4v){0.f, 0.f, 0.f, 0.f};
            compute_batch(0, raw, acc);
            float rcur[2][4];
            if (EPI == EPI_RES || EPI == EPI_AFFINE) {
#pragma unroll
                for (int dv = 0; dv < 2; ++dv)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        rcur[dv][r] = rnext[dv][r];
            }
            const int next = tile + gridDim.x;
            const Geo gn = geo_of(next);
            if (next < a.numTiles) {
                load_batch(gn, 0, raw);
                if (EPI == EPI_RES || (EPI == EPI_AFFINE && a.res))
                    load_res(gn, rnext);
            }
            __builtin_amdgcn_sched_barrier(0);
            finish_tile(g, acc, rcur);
            g = gn;
        }
    } else {
        for (int tile = blockIdx.x; tile < a.numTiles; tile += gridDim.x) {
            const Geo g = geo_of(tile);
            float4v acc[2][4];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[t][r] = (float4v){0.f, 0.f, 0.f, 0.f};
            float rr[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
            if (EPI == EPI_RES || (EPI == EPI_AFFINE && a.res))
                load_res(g, rr);
            for (int u0 = 0; u0 < KSWp; u0 += U) {
                PvRaw<PRO> raw[U];
                load_batch(g, u0, raw);
                __builtin_amdgcn_sched_barrier(0);
                compute_batch(u0, raw, acc);
            }
            finish_tile(g, acc, rr);
        }
    }
    if (EPI == EPI_STATS) {
#pragma unroll
        for (int dv = 0; dv < 2; ++dv) {
            const float s = row16_sum(ssum[dv]);
            const float s2 = row16_sum(ssq[dv]);
            const int m = 16 * tOwn + 4 * kk + vOwn + dv;
            if (j == 0 && m < a.M) {
                a.psum[(size_t)m * a.NP + blockIdx.x] = s;
                a.psq[(size_t)m * a.NP + blockIdx.x] = s2;
            }
        }
        // slots of workgroups that were not launched contribute nothing
        if (blockIdx.x == 0) {
            const int extra = a.NP - (int)gridDim.x;
            for (int idx = threadIdx.x; idx < a.M * extra; idx += 256) {
                const int m = idx / extra, slot = (int)gridDim.x + (idx - m * extra);
                a.psum[(size_t)m * a.NP + slot] = 0.f;
                a.psq[(size_t)m * a.NP + slot] = 0.f;
            }
        }
    }
}

// ---- dispatch ---------------------------------------------------------------------------------

// At most `cap` workgroups, each taking the same number of tiles (up to rounding): 1024 for
// conv_pr, 512 for conv_pe (measured on the 24 -> 144 channel, 100 k pixel layer: 392 workgroups
// of four tiles 23.4 us; 784 of two 24.5; 523 of three 26.3; 314 of five 26.4; 262 of six 28),
// 1024 and 2048 for conv_pe workgroups of two and of one wavefront (32 -> 16 channels, 803 k
// pixels: 75 us with 512 workgroups, 65 with 1024, 49 with 1536, 43 with 2048, 44 with 3072;
// 16 -> 96 channels: 106 us with 256, 85 with 512, 83 with 768, 79 with 1024, 86 with 1536).
static int pv_grid(int numTiles, int kind, int M)
{
    // conv_pe: a workgroup has one wavefront per 48 output channels, so a narrow output gets
    // more workgroups for the same number of wavefronts
    const int waves = ((M + 15) / 16 + kPeTT - 1) / kPeTT;
    const int pe_cap = waves >= 3 ? 512 : 2048 / waves;
    const int cap = kind == 1 ? pe_cap : 1024;
    if (numTiles <= cap)
        return numTiles < 1 ? 1 : numTiles;
    const int per = (numTiles + cap - 1) / cap;
    return (numTiles + per - 1) / per;
}

// Batch size and padded per-wavefront share (in input-channel quads) of conv_pr.
static void conv_pr_shape(int K, int *U, int *KSWp)
{
    const int ks4 = (K + 3) / 4, ksw = (ks4 + 3) / 4;
    const int p3 = (ksw + 2) / 3 * 3;
    *KSWp = p3;
    *U = (p3 % 9 == 0) ? 9 : (p3 % 6 == 0) ? 6 : 3;
}

static size_t conv_pr_lds(int K)
{
    int U, kswp;
    conv_pr_shape(K, &U, &kswp);
    const int ks4p = 4 * kswp;
    return sizeof(float) * ((size_t)12 * ks4p + 16 * 8 * 64 + (size_t)ks4p * 2 * 64);
}

// Which register-direct kernel covers (M, K, HW), if any: 1 = conv_pe, 2 = conv_pr, 0 = none.
int wave_conv_kind(int M, int K, int HW)
{
    if (HW % 4 != 0)
        return 0;
    if (K <= 40 && M <= 16 * kPeTT * kPeMaxWaves)
        return 1;
    if (M <= 32 && conv_pr_lds(K) <= 60 * 1024)
        return 2;
    return 0;
}

int wave_conv_num_partials(int kind, int N, int M, int HW)
{
    return pv_grid((int)(((long long)N * HW + 63) / 64), kind, M);
}

template <typename T, int PRO, int EPI>
static hipError_t launch_pe(const PvArgs &a, int grid, hipStream_t st)
{
    const int ks4 = (a.K + 3) / 4;
    const int waves = ((a.M + 15) / 16 + kPeTT - 1) / kPeTT;
#define MBK_E(KS4)                                                                                \
    if (ks4 <= KS4) {                                                                             \
        hipLaunchKernelGGL((conv_pe_kernel<T, KS4, PRO, EPI>), dim3(grid), dim3(64 * waves), 0, st, \
                           a);                                                                    \
        return hipGetLastError();                                                                 \
    }
    MBK_E(4)
    MBK_E(6)
    MBK_E(8)
    MBK_E(10)
#undef MBK_E
    return hipErrorInvalidValue;
}

// conv_pr workgroups are long (two barriers per tile), so a second wave of workgroups that
// starts when the first finishes would double the kernel's duration: launch no more than
// can be resident at once and let them stride over the tiles.  Partial-sum slots beyond the
// launched grid are zeroed by workgroup 0.
static int device_cu_count()
{
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess)
        (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    return cus > 0 ? cus : 256;
}

template <typename T, int PRO, int EPI>
static hipError_t launch_pr(PvArgs a, int grid, hipStream_t st)
{
    int U, kswp;
    conv_pr_shape(a.K, &U, &kswp);
    const size_t lds = conv_pr_lds(a.K);
#define MBK_PR(UU)                                                                                \
    if (U == UU) {                                                                                \
        auto kern = conv_pr_kernel<T, PRO, EPI, UU>;                                              \
        int per_cu = 0;                                                                           \
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 256, lds) != hipSuccess || \
            per_cu < 1)                                                                           \
            per_cu = 1;                                                                           \
        const int resident = per_cu * device_cu_count();                                          \
        if (grid > resident)                                                                      \
            grid = resident;                                                                      \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, a, kswp);                        \
        return hipGetLastError();                                                                 \
    }
    MBK_PR(9)
    MBK_PR(6)
    MBK_PR(3)
#undef MBK_PR
    return hipErrorInvalidValue;
}

template <typename T>
static hipError_t pv_dispatch(const PvArgs &a, int kind, int pro, int epi, int grid, hipStream_t st)
{
#define MBK_CASE(P, E)                                                                            \
    if (pro == P && epi == E)                                                                     \
        return kind == 1 ? launch_pe<T, P, E>(a, grid, st) : launch_pr<T, P, E>(a, grid, st);
    MBK_CASE(PRO_NONE, EPI_STATS)
    MBK_CASE(PRO_BNSWISH_GATE, EPI_STATS)
    MBK_CASE(PRO_BNBWD, EPI_NONE)
    MBK_CASE(PRO_BNBWD, EPI_RES)
#undef MBK_CASE
    if (kind == 2 && pro == PRO_BNSWISH_GATE && epi == EPI_AFFINE)
        return launch_pr<T, PRO_BNSWISH_GATE, EPI_AFFINE>(a, grid, st);
    return hipErrorNotSupported;
}

hipError_t launch_wave_conv1x1(bool bf16, int kind, int N, int M, int K, int HW, const void *w,
                               int sAm, int sAk, const Operand &B, void *out, int epi,
                               const void *res, float *psum, float *psq, hipStream_t st)
{
    PvArgs a;
    a.N = N;
    a.M = M;
    a.K = K;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    a.numTiles = (int)((a.Q + 63u) / 64u);
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
    const int grid = pv_grid(a.numTiles, kind, M);
    a.NP = grid;
    return bf16 ? pv_dispatch<bf16_t>(a, kind, B.pro, epi, grid, st)
                : pv_dispatch<float>(a, kind, B.pro, epi, grid, st);
}

} // namespace mbk
