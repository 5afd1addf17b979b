// bf16 storage on the bf16 matrix cores: 1x1 convolutions and weight gradients for the wide
// blocks when activations and conv weights are stored as bf16 (benchmark config 3).
//
// Same decomposition as kernels_big.hip (flattened batch, 64-pixel output tiles per workgroup of
// four wavefronts, two LDS buffers fed from a two-slot register ring, fixed-order split
// reductions), but the operands are kept as bf16 in LDS and contracted with
// v_mfma_f32_32x32x16_bf16 (fp32 accumulation), which is 16 times the fp32 MFMA rate and, unlike
// the fp32 MFMA, runs beside the vector ALU: these kernels cost what their staging arithmetic and
// HBM traffic cost.  The elementwise prologue (Swish(BN(.))*gate or the BN-backward expression)
// is evaluated in fp32 and rounded to bf16 once, on the way into LDS.
//
// Operand layout of the instruction (checked on the device): lane l holds, of A, row l%32 and the
// eight contraction indices 8*(l/32)..+7; of B, column l%32 and the same eight indices.  Both
// LDS tiles are therefore stored [row or column][k] with k contiguous, pitch BK+8 elements
// (80 or 144 bytes: 16-byte aligned rows whose 16-byte reads fall on distinct banks).
#include "mbconv_dev.h"
#include "mbconv_launch.h"

namespace mbk {

typedef float float16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct BfOperand {
    const bf16_t *p0, *p1;
    const float *c0, *c1, *c2, *gate;
};

__device__ __forceinline__ uint32_t bf_pack2(float lo, float hi)
{
    return bf16_pack2(lo, hi);
}
__device__ __forceinline__ void bf_unpack4(uint2 t, float (&v)[4])
{
    v[0] = bf16_bits_to_float(t.x & 0xffffu);
    v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = bf16_bits_to_float(t.y & 0xffffu);
    v[3] = __uint_as_float(t.y & 0xffff0000u);
}
template <int PRO>
__device__ __forceinline__ float bf_apply(float v0, float v1, float k0, float k1, float k2)
{
    if (PRO == PRO_NONE)
        return v0;
    if (PRO == PRO_BNSWISH_GATE)
        return actf(fmaf(v0, k0, k1)) * k2;
    return fmaf(k0, v0, fmaf(k1, v1, k2));
}
// Column of contraction index k in row `row` of the activation tile: the four 16-byte groups of
// a row are permuted by bits 4-5 of the row, so that the transposing stores of a wavefront
// (one 32-bit k pair to each of 16 rows that are four apart) fall on distinct banks; the
// 16-byte fragment reads of 16 consecutive rows stay conflict-free.
__device__ __forceinline__ int bf_bcol(int row, int k)
{
    return ((((k >> 3) ^ (row >> 4)) & 3) << 3) + (k & 7);
}
__device__ __forceinline__ bf16x8 bf_lds8(const uint16_t *p)
{
    return *reinterpret_cast<const bf16x8 *>(p);
}

// ---- convolution ---------------------------------------------------------------------------
struct BfConvArgs {
    int M, K, HW;
    uint32_t Q;
    FastDiv divHW;
    const bf16_t *w;
    int sAm, sAk;
    BfOperand B;
    bf16_t *out;
    const bf16_t *res;
    float *psum, *psq;
    int QT, MT;
    float *partial;
    int chunksPerSplit;
};

// out[n,m,pix] = sum_k A(m,k) * op(B)[n,k,pix].  Requirements (checked by the host):
// K % 8 == 0, M % 8 == 0, HW % 4 == 0, one of sAm/sAk equal to 1.
// A workgroup owns 64*WM output rows and 64 pixels; each of its four wavefronts 32*WM rows by
// 32 pixels (WM accumulator tiles).  The activation tile is staged (and sent through its
// prologue) once per workgroup, so a taller tile divides the prologue arithmetic per output:
// on the bf16 matrix cores that arithmetic, not the MFMAs, is what these kernels cost.
template <int PRO, int EPI, int WM>
__global__ __launch_bounds__(256) void conv_bf_kernel(BfConvArgs a)
{
    constexpr int BM = 64 * WM, BP = 64, BK = 32, PK = BK + 8, PC = BP + 4;
    // one LDS block: the two operand buffers during the contraction, one 64-row slab of the
    // fp32 output tile at a time after it
    constexpr int kOperandBytes = 2 * (BM + BP) * PK * 2, kTileBytes = 64 * PC * 4;
    __shared__ __attribute__((aligned(16))) unsigned char smem[kOperandBytes > kTileBytes ? kOperandBytes : kTileBytes];
    uint16_t(*As)[BM][PK] = reinterpret_cast<uint16_t(*)[BM][PK]>(smem);
    uint16_t(*Bs)[BP][PK] = reinterpret_cast<uint16_t(*)[BP][PK]>(smem + 2 * BM * PK * 2);
    float(*Ct)[PC] = reinterpret_cast<float(*)[PC]>(smem);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wp = wave & 1;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int qt = (slot / a.MT) * 8 + xcd, mt = slot % a.MT;
    if (qt >= a.QT)
        return;
    const int m0 = mt * BM;
    const uint32_t q0 = (uint32_t)qt * BP;
    const bool kcontig = a.sAk == 1;

    // Staged chunks live in a ring of two register slots: chunk j is loaded during iteration
    // j-2 and written to LDS at the end of iteration j-1.  All loads are unconditional (indices
    // clamped into the tensor, the chunk index to the last chunk) and validity is an AND mask
    // applied on the way into LDS: no branch and no use of loaded data sits between a load and
    // the MFMAs it should overlap, so the compiler's wait counts stay exact.
    //
    // A staging, 64 rows per pass.  k-contiguous weights: thread -> (row tid/4, eight k at
    // 8*(tid%4)), a straight 16-byte copy.  m-contiguous weights (data gradients): thread ->
    // (k = tid%32, eight rows at 8*(tid/32)), transposed with 2-byte LDS stores.
    uint4 ra[2][WM];
    uint32_t raok[2][WM];
    auto load_a = [&](int slot_, int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            if (kcontig) {
                const int m = m0 + 64 * i + (tid >> 2), k = k0 + 8 * (tid & 3);
                raok[slot_][i] = (m < a.M && k < a.K) ? 0xffffffffu : 0u;
                ra[slot_][i] = *reinterpret_cast<const uint4 *>(a.w + (size_t)min(m, a.M - 1) * a.sAm + min(k, a.K - 8));
            } else {
                const int k = k0 + (tid & 31), m = m0 + 64 * i + 8 * (tid >> 5);
                raok[slot_][i] = (m < a.M && k < a.K) ? 0xffffffffu : 0u;
                ra[slot_][i] = *reinterpret_cast<const uint4 *>(a.w + (size_t)min(k, a.K - 1) * a.sAk + min(m, a.M - 8));
            }
        }
    };
    auto store_a = [&](int slot_, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const uint32_t mk = raok[slot_][i];
            const uint4 v = make_uint4(ra[slot_][i].x & mk, ra[slot_][i].y & mk, ra[slot_][i].z & mk, ra[slot_][i].w & mk);
            if (kcontig) {
                *reinterpret_cast<uint4 *>(&As[buf][64 * i + (tid >> 2)][8 * (tid & 3)]) = v;
            } else {
                const int kk = tid & 31, mm = 64 * i + 8 * (tid >> 5);
                As[buf][mm + 0][kk] = (uint16_t)(v.x & 0xffffu);
                As[buf][mm + 1][kk] = (uint16_t)(v.x >> 16);
                As[buf][mm + 2][kk] = (uint16_t)(v.y & 0xffffu);
                As[buf][mm + 3][kk] = (uint16_t)(v.y >> 16);
                As[buf][mm + 4][kk] = (uint16_t)(v.z & 0xffffu);
                As[buf][mm + 5][kk] = (uint16_t)(v.z >> 16);
                As[buf][mm + 6][kk] = (uint16_t)(v.w & 0xffffu);
                As[buf][mm + 7][kk] = (uint16_t)(v.w >> 16);
            }
        }
    };

    // B staging: thread -> (four pixels at 4*(tid%16), channel pair 2*(tid/16)); the pair of a
    // pixel is packed into one 32-bit LDS store.  The pixel run is the same for every chunk.
    const int pg = tid & 15, kp = tid >> 4;
    const uint32_t qb = q0 + 4u * pg;
    const bool bvalid = qb < a.Q;
    const uint32_t bn = bvalid ? fdiv(qb, a.divHW) : 0u;
    const size_t bbase = (size_t)bn * a.K * a.HW + (bvalid ? qb - bn * (uint32_t)a.HW : 0u);
    uint2 rb0[2][2], rb1[2][2];
    float bk0[2][2], bk1[2][2], bk2[2][2];
    uint32_t rbok[2][2];
    auto load_b = [&](int slot_, int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int k = k0 + 2 * kp + i, kc = min(k, a.K - 1);
            rbok[slot_][i] = (bvalid && k < a.K) ? 0xffffffffu : 0u;
            rb0[slot_][i] = *reinterpret_cast<const uint2 *>(a.B.p0 + bbase + (size_t)kc * a.HW);
            if (PRO == PRO_BNBWD)
                rb1[slot_][i] = *reinterpret_cast<const uint2 *>(a.B.p1 + bbase + (size_t)kc * a.HW);
            if (PRO != PRO_NONE) {
                bk0[slot_][i] = a.B.c0[kc];
                bk1[slot_][i] = a.B.c1[kc];
                bk2[slot_][i] = PRO == PRO_BNBWD ? a.B.c2[kc] : a.B.gate[(size_t)bn * a.K + kc];
            }
        }
    };
    auto store_b = [&](int slot_, int buf) __attribute__((always_inline)) {
        if (PRO == PRO_NONE) {
            // no arithmetic: re-pair the halves of the two channel rows
            const uint2 lo = make_uint2(rb0[slot_][0].x & rbok[slot_][0], rb0[slot_][0].y & rbok[slot_][0]);
            const uint2 hi = make_uint2(rb0[slot_][1].x & rbok[slot_][1], rb0[slot_][1].y & rbok[slot_][1]);
            *reinterpret_cast<uint32_t *>(&Bs[buf][4 * pg + 0][bf_bcol(4 * pg, 2 * kp)]) = (lo.x & 0xffffu) | (hi.x << 16);
            *reinterpret_cast<uint32_t *>(&Bs[buf][4 * pg + 1][bf_bcol(4 * pg, 2 * kp)]) = (lo.x >> 16) | (hi.x & 0xffff0000u);
            *reinterpret_cast<uint32_t *>(&Bs[buf][4 * pg + 2][bf_bcol(4 * pg, 2 * kp)]) = (lo.y & 0xffffu) | (hi.y << 16);
            *reinterpret_cast<uint32_t *>(&Bs[buf][4 * pg + 3][bf_bcol(4 * pg, 2 * kp)]) = (lo.y >> 16) | (hi.y & 0xffff0000u);
            return;
        }
        float v[2][4];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            float x0[4], x1[4] = {0.f, 0.f, 0.f, 0.f};
            bf_unpack4(rb0[slot_][i], x0);
            if (PRO == PRO_BNBWD)
                bf_unpack4(rb1[slot_][i], x1);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                v[i][r] = and_mask(bf_apply<PRO>(x0[r], x1[r], bk0[slot_][i], bk1[slot_][i], bk2[slot_][i]),
                                   rbok[slot_][i]);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
            *reinterpret_cast<uint32_t *>(&Bs[buf][4 * pg + r][bf_bcol(4 * pg, 2 * kp)]) = bf_pack2(v[0][r], v[1][r]);
    };

    float16v acc[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            acc[i][r] = 0.f;

    int cbeg = 0, cend = (a.K + BK - 1) / BK;
    if (EPI == EPI_PARTIAL) {
        cbeg = blockIdx.y * a.chunksPerSplit;
        cend = min(cbeg + a.chunksPerSplit, cend);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int cl = min(cbeg + u, cend - 1);
        load_a(u, cl * BK);
        load_b(u, cl * BK);
    }
    store_a(0, 0);
    store_b(0, 0);
    __syncthreads();
    auto step = [&](int u, int cc) __attribute__((always_inline)) {
        const int buf = (cc - cbeg) & 1;
        const int cl = min(cc + 2, cend - 1); // slot u is free: its chunk went to LDS last iteration
        load_a(u, cl * BK);
        load_b(u, cl * BK);
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            const bf16x8 bv = bf_lds8(&Bs[buf][wp * 32 + (lane & 31)][bf_bcol(wp * 32 + (lane & 31), 16 * s + 8 * (lane >> 5))]);
#pragma unroll
            for (int i = 0; i < WM; ++i) {
                const bf16x8 av = bf_lds8(&As[buf][wm * 32 * WM + 32 * i + (lane & 31)][16 * s + 8 * (lane >> 5)]);
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[i], 0, 0, 0);
            }
        }
        store_a(u ^ 1, buf ^ 1); // the repeated last chunk is stored but never consumed
        store_b(u ^ 1, buf ^ 1);
        __syncthreads();
    };
    {
        const int turns = (cend - cbeg) / 2;
        int cc = cbeg;
        for (int g = 0; g < turns; ++g) {
            step(0, cc);
            step(1, cc + 1);
            cc += 2;
        }
        if ((cend - cbeg) & 1) // uniform over the workgroup
            step(0, cc);
    }

    // epilogue: register r of lane l is row 8*(r/4)+4*(l/32)+r%4, column l%32
    if (EPI == EPI_PARTIAL) {
        const uint32_t q = q0 + wp * 32 + (lane & 31);
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 32 * WM + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (q < a.Q && m < a.M)
                    a.partial[((size_t)blockIdx.y * a.M + m) * a.Q + q] = acc[i][r];
            }
        return;
    }
    // The tile goes through LDS, 64 rows at a time, so that a thread ends up with four
    // consecutive pixels of a row: 8-byte global accesses, 128 contiguous bytes per row and
    // instruction, one pixel-index division per thread, and the BN statistics of a row reduced
    // inside 16 lanes.
    const uint32_t q = q0 + 4u * pg; // pg = tid % 16: the same pixel run as in the staging
    const bool valid = q < a.Q;
    const uint32_t n = valid ? fdiv(q, a.divHW) : 0u;
    const uint32_t pix = valid ? q - n * (uint32_t)a.HW : 0u;
#pragma unroll
    for (int h = 0; h < WM; ++h) {
        if (h)
            __syncthreads(); // the previous slab has been read
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const int r0 = wm * 32 * WM + 32 * i; // first row of this accumulator tile
            if (r0 / 64 == h) {                   // wave-uniform
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    Ct[(r0 & 63) + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)][wp * 32 + (lane & 31)] = acc[i][r];
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = (tid >> 4) + 16 * i, m = m0 + 64 * h + row;
            const float4 c4 = *reinterpret_cast<const float4 *>(&Ct[row][4 * pg]);
            float v[4] = {c4.x, c4.y, c4.z, c4.w};
            const bool ok = valid && m < a.M;
            const size_t idx = ((size_t)n * a.M + (ok ? m : 0)) * a.HW + pix;
            if (EPI == EPI_RES) {
                float rr[4];
                bf_unpack4(*reinterpret_cast<const uint2 *>(a.res + idx), rr);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    v[r] += rr[r];
            }
            if (EPI == EPI_AFFINE) { // psum / psq carry the row's scale and shift
                const float osc = a.psum[ok ? m : 0], osh = a.psq[ok ? m : 0];
                float rr[4] = {0.f, 0.f, 0.f, 0.f};
                if (a.res)
                    bf_unpack4(*reinterpret_cast<const uint2 *>(a.res + idx), rr);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    v[r] = fmaf(v[r], osc, osh) + rr[r];
            }
            const uint2 packed = make_uint2(bf_pack2(v[0], v[1]), bf_pack2(v[2], v[3]));
            if (ok)
                *reinterpret_cast<uint2 *>(a.out + idx) = packed;
            if (EPI == EPI_STATS) {
                float sv[4], s1 = 0.f, s2 = 0.f;
                bf_unpack4(packed, sv);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    s1 += ok ? sv[r] : 0.f;
                    s2 = fmaf(ok ? sv[r] : 0.f, sv[r], s2);
                }
                s1 = row16_sum(s1);
                s2 = row16_sum(s2);
                if (pg == 0 && m < a.M) {
                    a.psum[(size_t)m * a.QT + qt] = s1;
                    a.psq[(size_t)m * a.QT + qt] = s2;
                }
            }
        }
    }
}

// second stage of a split convolution (see splitk_finish_kernel in kernels_big.hip)
template <int EPI>
__global__ __launch_bounds__(256) void bf_splitk_finish_kernel(const float *__restrict__ partial, int S,
                                                               int M, uint32_t Q, FastDiv divHW, int HW,
                                                               bf16_t *out, const bf16_t *res,
                                                               float *psum, float *psq, int NT)
{
    __shared__ float red[2][4];
    const int m = blockIdx.y, tid = threadIdx.x;
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t q = blockIdx.x * 1024u + 256u * i + tid;
        if (q < Q) {
            float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
            const float *src = partial + (size_t)m * Q + q;
            const size_t step = (size_t)M * Q;
            int s = 0;
            for (; s + 3 < S; s += 4) {
                v0 += src[(size_t)s * step];
                v1 += src[(size_t)(s + 1) * step];
                v2 += src[(size_t)(s + 2) * step];
                v3 += src[(size_t)(s + 3) * step];
            }
            for (; s < S; ++s)
                v0 += src[(size_t)s * step];
            float v = (v0 + v1) + (v2 + v3);
            const uint32_t n = fdiv(q, divHW), pix = q - n * (uint32_t)HW;
            const size_t idx = ((size_t)n * M + m) * HW + pix;
            if (EPI == EPI_RES)
                v += ld<bf16_t>(res, idx);
            st<bf16_t>(out, idx, v);
            if (EPI == EPI_STATS) {
                const float sv = as_stored<bf16_t>(v);
                s1 += sv;
                s2 = fmaf(sv, sv, s2);
            }
        }
    }
    if (EPI == EPI_STATS) {
        s1 = wave_sum(s1);
        s2 = wave_sum(s2);
        if ((tid & 63) == 0) {
            red[0][tid >> 6] = s1;
            red[1][tid >> 6] = s2;
        }
        __syncthreads();
        if (tid == 0) {
            psum[(size_t)m * NT + blockIdx.x] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
            psq[(size_t)m * NT + blockIdx.x] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
        }
    }
}

// Plan: 64x64 tiles; the contraction is split when the tiles alone cannot fill the chip.
bool bf_conv_plan(int N, int M, int K, int HW, int *qtiles, int *splits)
{
    const long long Q = (long long)N * HW;
    if (K % 8 != 0 || M % 8 != 0 || HW % 4 != 0 || Q >= (1ll << 31) || K < 32)
        return false;
    *qtiles = (int)((Q + 63) / 64);
    *splits = 1;
    const long long tiles = (long long)*qtiles * ((M + 63) / 64);
    const int chunks = (K + 31) / 32;
    if (tiles < 384 && chunks >= 8) {
        long long s = (768 + tiles - 1) / tiles;
        if (s > chunks / 2)
            s = chunks / 2;
        if (s > 16)
            s = 16;
        const int per = (int)((chunks + s - 1) / s);
        *splits = (chunks + per - 1) / per;
        if (*splits > 1)
            *qtiles = (int)((Q + 1023) / 1024);
    }
    return true;
}

// Rows per workgroup (in units of 64) of an unsplit convolution.  Measured on the 14x14 blocks
// (112 <-> 672 channels, batch 128): 128 rows beat 64 for both the 112-row and the 672-row
// outputs (the activation tile and its prologue are staged half as often), 256 rows lose again
// (too few workgroups, long epilogue).
static int bf_conv_rows(int N, int M, int HW)
{
    const long long qtiles = ((long long)N * HW + 63) / 64;
    return (M > 64 && qtiles * ((M + 127) / 128) >= 256) ? 2 : 1;
}

size_t bf_conv_splitk_floats(int N, int M, int K, int HW)
{
    int qtiles, splits;
    if (!bf_conv_plan(N, M, K, HW, &qtiles, &splits) || splits == 1)
        return 0;
    return (size_t)splits * M * N * HW;
}

hipError_t launch_bf_conv1x1(int N, int M, int K, int HW, const void *w, int sAm, int sAk,
                             const Operand &B, void *out, int epi, const void *res, float *psum,
                             float *psq, float *splitk_ws, hipStream_t st)
{
    int qtiles, splits;
    if (!bf_conv_plan(N, M, K, HW, &qtiles, &splits) || (sAm != 1 && sAk != 1))
        return hipErrorInvalidValue;
    if (splits > 1 && !splitk_ws)
        return hipErrorInvalidValue;
    BfConvArgs a;
    a.M = M;
    a.K = K;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    a.divHW = make_div((uint32_t)HW);
    a.w = (const bf16_t *)w;
    a.sAm = sAm;
    a.sAk = sAk;
    a.B.p0 = (const bf16_t *)B.p0;
    a.B.p1 = (const bf16_t *)B.p1;
    a.B.c0 = B.c0;
    a.B.c1 = B.c1;
    a.B.c2 = B.c2;
    a.B.gate = B.gate;
    a.out = (bf16_t *)out;
    a.res = (const bf16_t *)res;
    a.psum = psum;
    a.psq = psq;
    const int wm = splits > 1 ? 1 : bf_conv_rows(N, M, HW);
    a.QT = (int)((a.Q + 63u) / 64u);
    a.MT = (M + 64 * wm - 1) / (64 * wm);
    a.partial = splitk_ws;
    const int chunks = (K + 31) / 32;
    a.chunksPerSplit = (chunks + splits - 1) / splits;
    dim3 grid((unsigned)(((a.QT + 7) / 8) * 8 * a.MT), (unsigned)splits);
    const int kepi = splits > 1 ? EPI_PARTIAL : epi;
    hipError_t e = hipErrorInvalidValue;
#define MBK_CASE(P, E, W)                                                                         \
    if (B.pro == P && kepi == E && wm == W) {                                                     \
        hipLaunchKernelGGL((conv_bf_kernel<P, E, W>), grid, dim3(256), 0, st, a);                 \
        e = hipGetLastError();                                                                    \
    }
#define MBK_ROWS(P, E) MBK_CASE(P, E, 1) MBK_CASE(P, E, 2)
    MBK_ROWS(PRO_NONE, EPI_STATS)
    MBK_ROWS(PRO_BNSWISH_GATE, EPI_STATS)
    MBK_ROWS(PRO_BNBWD, EPI_NONE)
    MBK_ROWS(PRO_BNBWD, EPI_RES)
    MBK_ROWS(PRO_BNSWISH_GATE, EPI_AFFINE)
    MBK_CASE(PRO_NONE, EPI_PARTIAL, 1)
    MBK_CASE(PRO_BNSWISH_GATE, EPI_PARTIAL, 1)
    MBK_CASE(PRO_BNBWD, EPI_PARTIAL, 1)
#undef MBK_ROWS
#undef MBK_CASE
    if (e != hipSuccess || splits == 1)
        return e;
    dim3 fgrid((unsigned)qtiles, (unsigned)M);
    const FastDiv dv = make_div((uint32_t)HW);
#define MBK_CASE(E)                                                                               \
    if (epi == E) {                                                                               \
        hipLaunchKernelGGL((bf_splitk_finish_kernel<E>), fgrid, dim3(256), 0, st, splitk_ws, splits, \
                           M, a.Q, dv, HW, a.out, a.res, psum, psq, qtiles);                      \
        return hipGetLastError();                                                                 \
    }
    MBK_CASE(EPI_NONE)
    MBK_CASE(EPI_STATS)
    MBK_CASE(EPI_RES)
#undef MBK_CASE
    return hipErrorInvalidValue;
}

// ---- weight gradient -------------------------------------------------------------------------
// dW[a,b] = sum_q op(U)[a,q] * op(V)[b,q]: both operands are pixel-contiguous, which is exactly
// the [row][k] layout the instruction wants, so the tiles go into LDS untransposed (8-byte runs
// of four pixels per thread).  64 pixels per chunk; the contraction is split over blockIdx.z.
struct BfWgradArgs {
    int Ma, Mb, HW;
    uint32_t Q;
    int chunksPerSplit; // chunks of 64 pixels
    int tilesA, tilesB, splits;
    FastDiv divHW;
    BfOperand U, V;
    float *partial;
};

// A workgroup owns 64*WA rows of U by 64*WB rows of V; each wavefront 32*WA by 32*WB.  A tile
// that spans all rows of the narrow operand stages the wide one (and evaluates its prologue)
// only once in the whole grid.
template <int PROU, int PROV, int WA, int WB>
__global__ __launch_bounds__(256) void wgrad_bf_kernel(BfWgradArgs a)
{
    constexpr int BA = 64 * WA, BB = 64 * WB, BQ = 64, PQ = BQ + 8;
    constexpr int NU = 4 * WA, NV = 4 * WB; // 16 rows per pass
    __shared__ __attribute__((aligned(16))) uint16_t Us[2][BA][PQ];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[2][BB][PQ];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wa = wave >> 1, wb = wave & 1;
    // workgroups that read the same pixels (all tiles of one split) run on the same XCD
    // (blockIdx.x mod 8), so the operand that several tiles share comes out of that XCD's L2
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int tiles = a.tilesA * a.tilesB;
    const int split = (slot / tiles) * 8 + xcd, tile = slot % tiles;
    if (split >= a.splits)
        return;
    const int a0 = (tile % a.tilesA) * BA, b0 = (tile / a.tilesA) * BB;
    const int numChunks = (int)((a.Q + BQ - 1) / BQ);
    const int cbeg = split * a.chunksPerSplit;
    const int cend = min(cbeg + a.chunksPerSplit, numChunks);

    const int qg = tid & 15, rrow = tid >> 4;
    float uk[NU][3], vk[NV][3];
    uint32_t umask[NU], vmask[NV];
#pragma unroll
    for (int i = 0; i < NU; ++i) {
        const int ra = a0 + rrow + 16 * i;
        umask[i] = ra < a.Ma ? 0xffffffffu : 0u;
        uk[i][0] = uk[i][1] = uk[i][2] = 0.f;
        if (PROU != PRO_NONE && ra < a.Ma) {
            uk[i][0] = a.U.c0[ra];
            uk[i][1] = a.U.c1[ra];
            if (PROU == PRO_BNBWD)
                uk[i][2] = a.U.c2[ra];
        }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int rb = b0 + rrow + 16 * i;
        vmask[i] = rb < a.Mb ? 0xffffffffu : 0u;
        vk[i][0] = vk[i][1] = vk[i][2] = 0.f;
        if (PROV != PRO_NONE && rb < a.Mb) {
            vk[i][0] = a.V.c0[rb];
            vk[i][1] = a.V.c1[rb];
            if (PROV == PRO_BNBWD)
                vk[i][2] = a.V.c2[rb];
        }
    }
    // Ring of two register slots (see conv_bf_kernel): unconditional clamped loads, validity as
    // an AND mask on the way into LDS.
    uint2 u0[2][NU], u1[2][NU], v0[2][NV], v1[2][NV];
    float ug[2][NU], vg[2][NV];
    uint32_t qmask[2];
    auto load = [&](int slot, int chunk) __attribute__((always_inline)) {
        const uint32_t q = (uint32_t)chunk * BQ + 4u * qg;
        const bool valid = q < a.Q;
        qmask[slot] = valid ? 0xffffffffu : 0u;
        const uint32_t qc = valid ? q : 0u;
        const uint32_t n = fdiv(qc, a.divHW);
        const uint32_t pix = qc - n * (uint32_t)a.HW;
#pragma unroll
        for (int i = 0; i < NU; ++i) {
            const int ra = min(a0 + rrow + 16 * i, a.Ma - 1);
            const size_t iu = ((size_t)n * a.Ma + ra) * a.HW + pix;
            u0[slot][i] = *reinterpret_cast<const uint2 *>(a.U.p0 + iu);
            if (PROU == PRO_BNBWD)
                u1[slot][i] = *reinterpret_cast<const uint2 *>(a.U.p1 + iu);
            if (PROU == PRO_BNSWISH_GATE)
                ug[slot][i] = a.U.gate[(size_t)n * a.Ma + ra];
        }
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int rb = min(b0 + rrow + 16 * i, a.Mb - 1);
            const size_t iv = ((size_t)n * a.Mb + rb) * a.HW + pix;
            v0[slot][i] = *reinterpret_cast<const uint2 *>(a.V.p0 + iv);
            if (PROV == PRO_BNBWD)
                v1[slot][i] = *reinterpret_cast<const uint2 *>(a.V.p1 + iv);
            if (PROV == PRO_BNSWISH_GATE)
                vg[slot][i] = a.V.gate[(size_t)n * a.Mb + rb];
        }
    };
    auto store = [&](int slot, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NU; ++i) {
            const int row = rrow + 16 * i;
            const uint32_t mk = qmask[slot] & umask[i];
            if (PROU == PRO_NONE) {
                *reinterpret_cast<uint2 *>(&Us[buf][row][4 * qg]) = make_uint2(u0[slot][i].x & mk, u0[slot][i].y & mk);
            } else {
                float x0[4], x1[4] = {0.f, 0.f, 0.f, 0.f}, y[4];
                bf_unpack4(u0[slot][i], x0);
                if (PROU == PRO_BNBWD)
                    bf_unpack4(u1[slot][i], x1);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    y[r] = and_mask(bf_apply<PROU>(x0[r], x1[r], uk[i][0], uk[i][1],
                                                   PROU == PRO_BNSWISH_GATE ? ug[slot][i] : uk[i][2]), mk);
                *reinterpret_cast<uint2 *>(&Us[buf][row][4 * qg]) =
                    make_uint2(bf_pack2(y[0], y[1]), bf_pack2(y[2], y[3]));
            }
        }
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int row = rrow + 16 * i;
            const uint32_t mk = qmask[slot] & vmask[i];
            if (PROV == PRO_NONE) {
                *reinterpret_cast<uint2 *>(&Vs[buf][row][4 * qg]) = make_uint2(v0[slot][i].x & mk, v0[slot][i].y & mk);
            } else {
                float x0[4], x1[4] = {0.f, 0.f, 0.f, 0.f}, y[4];
                bf_unpack4(v0[slot][i], x0);
                if (PROV == PRO_BNBWD)
                    bf_unpack4(v1[slot][i], x1);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    y[r] = and_mask(bf_apply<PROV>(x0[r], x1[r], vk[i][0], vk[i][1],
                                                   PROV == PRO_BNSWISH_GATE ? vg[slot][i] : vk[i][2]), mk);
                *reinterpret_cast<uint2 *>(&Vs[buf][row][4 * qg]) =
                    make_uint2(bf_pack2(y[0], y[1]), bf_pack2(y[2], y[3]));
            }
        }
    };

    float16v acc[WA][WB];
#pragma unroll
    for (int i = 0; i < WA; ++i)
#pragma unroll
        for (int j = 0; j < WB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0.f;
    if (cbeg < cend) { // uniform over the workgroup; an empty split writes zeros
        load(0, cbeg);
        load(1, min(cbeg + 1, cend - 1));
        store(0, 0);
        __syncthreads();
        auto step = [&](int u, int cc) __attribute__((always_inline)) {
            const int buf = (cc - cbeg) & 1;
            load(u, min(cc + 2, cend - 1)); // slot u is free: its chunk went to LDS last iteration
#pragma unroll
            for (int s = 0; s < BQ / 16; ++s) {
                bf16x8 av[WA], bv[WB];
#pragma unroll
                for (int i = 0; i < WA; ++i)
                    av[i] = bf_lds8(&Us[buf][wa * 32 * WA + 32 * i + (lane & 31)][16 * s + 8 * (lane >> 5)]);
#pragma unroll
                for (int j = 0; j < WB; ++j)
                    bv[j] = bf_lds8(&Vs[buf][wb * 32 * WB + 32 * j + (lane & 31)][16 * s + 8 * (lane >> 5)]);
#pragma unroll
                for (int i = 0; i < WA; ++i)
#pragma unroll
                    for (int j = 0; j < WB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
            }
            store(u ^ 1, buf ^ 1); // the repeated last chunk is stored but never consumed
            __syncthreads();
        };
        const int turns = (cend - cbeg) / 2;
        int cc = cbeg;
        for (int g = 0; g < turns; ++g) {
            step(0, cc);
            step(1, cc + 1);
            cc += 2;
        }
        if ((cend - cbeg) & 1)
            step(0, cc);
    }
    float *dst = a.partial + (size_t)split * a.Ma * a.Mb;
#pragma unroll
    for (int i = 0; i < WA; ++i)
#pragma unroll
        for (int j = 0; j < WB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ai = a0 + wa * 32 * WA + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const int bi = b0 + wb * 32 * WB + 32 * j + (lane & 31);
                if (ai < a.Ma && bi < a.Mb)
                    dst[(size_t)ai * a.Mb + bi] = acc[i][j][r];
            }
}

// Tile shape.  A narrow second operand (65-128 rows: the block input of the expansion weight
// gradient) is covered by one 128-row tile, so the wide first operand is staged once in the whole
// grid (measured 45 against 54 us on 672 x 112 channels, batch 128, 14x14); the mirrored shape
// (narrow first operand) measured slower than 64 x 64 and is not used.
static void bf_wgrad_tile(int Ma, int Mb, int *wa, int *wb)
{
    (void)Ma;
    *wa = 1;
    *wb = (Mb > 64 && Mb <= 128) ? 2 : 1;
}

bool bf_wgrad_plan(int Ma, int Mb, int N, int HW, int *splits)
{
    const long long Q = (long long)N * HW;
    if (HW % 4 != 0 || Q >= (1ll << 31))
        return false;
    int wa, wb;
    bf_wgrad_tile(Ma, Mb, &wa, &wb);
    const long long tiles = (long long)((Ma + 64 * wa - 1) / (64 * wa)) * ((Mb + 64 * wb - 1) / (64 * wb));
    const long long chunks = (Q + 63) / 64;
    long long s = (640 + tiles - 1) / tiles;
    const long long smax = (chunks + 3) / 4; // at least four chunks per split
    if (s > smax)
        s = smax;
    if (s < 1)
        s = 1;
    const long long per = (chunks + s - 1) / s;
    *splits = (int)((chunks + per - 1) / per);
    return true;
}

hipError_t launch_bf_wgrad(int N, int Ma, int Mb, int HW, const Operand &U, const Operand &V,
                           float *partial, int *splits_out, hipStream_t st)
{
    int splits;
    if (!bf_wgrad_plan(Ma, Mb, N, HW, &splits))
        return hipErrorInvalidValue;
    BfWgradArgs a;
    a.Ma = Ma;
    a.Mb = Mb;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    const int chunks = (int)((a.Q + 63u) / 64u);
    a.chunksPerSplit = (chunks + splits - 1) / splits;
    a.divHW = make_div((uint32_t)HW);
    a.U.p0 = (const bf16_t *)U.p0;
    a.U.p1 = (const bf16_t *)U.p1;
    a.U.c0 = U.c0;
    a.U.c1 = U.c1;
    a.U.c2 = U.c2;
    a.U.gate = U.gate;
    a.V.p0 = (const bf16_t *)V.p0;
    a.V.p1 = (const bf16_t *)V.p1;
    a.V.c0 = V.c0;
    a.V.c1 = V.c1;
    a.V.c2 = V.c2;
    a.V.gate = V.gate;
    a.partial = partial;
    *splits_out = splits;
    int wa, wb;
    bf_wgrad_tile(Ma, Mb, &wa, &wb);
    a.tilesA = (Ma + 64 * wa - 1) / (64 * wa);
    a.tilesB = (Mb + 64 * wb - 1) / (64 * wb);
    a.splits = splits;
    dim3 grid((unsigned)(((splits + 7) / 8) * 8 * a.tilesA * a.tilesB));
#define MBK_CASE(PU, PV, A, B)                                                                    \
    if (U.pro == PU && V.pro == PV && wa == A && wb == B) {                                       \
        hipLaunchKernelGGL((wgrad_bf_kernel<PU, PV, A, B>), grid, dim3(256), 0, st, a);           \
        return hipGetLastError();                                                                 \
    }
#define MBK_TILES(PU, PV) MBK_CASE(PU, PV, 1, 1) MBK_CASE(PU, PV, 1, 2)
    MBK_TILES(PRO_BNBWD, PRO_NONE)
    MBK_TILES(PRO_BNBWD, PRO_BNSWISH_GATE)
#undef MBK_TILES
#undef MBK_CASE
    return hipErrorInvalidValue;
}

} // namespace mbk
