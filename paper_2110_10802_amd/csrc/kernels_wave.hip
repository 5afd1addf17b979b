// Register-direct weight gradients of the 1x1 convolutions for the HBM-bound ("skinny") shapes.
//
// MFMA used: v_mfma_f32_32x32x2_f32, C[i][j] += sum_k A[i][k]*B[k][j] with
//   A: lane l holds A[i = l%32][k = l/32],  B: lane l holds B[k = l/32][j = l%32],
//   C: lane l, register r holds C[i = 8*(r/4) + 4*(l/32) + r%4][j = l%32].
//
// wgrad_cl, "channel-lane" form: dW[a][b] = sum_pix U[a][pix]*V[b][pix].  The contraction
// runs over pixels, so a lane owns a channel (A: i = a, B: j = b) and loads float4 runs of its
// channel's pixels (16 bytes per lane: a dword-per-lane stream reaches under half the
// bandwidth on this chip); the two lane halves and the four vector elements enumerate the
// contraction index.  The operands' elementwise prologues (BN backward, Swish(BN(.))*gate)
// run on the registers between load and MFMA.  Workgroups split the pixel range; partial
// tiles are summed in a fixed order by reduce_splits (no atomics: the paper's map-fission
// step, section "Guided Optimization Case Study: EfficientNet").
#include "mbconv_dev.h"
#include "mbconv_launch.h"

namespace mbk {

typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));

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
            v[r] = actf(fmaf(v[r], k0, k1)) * g;
    }
}

template <typename T, int MTA, int PROU, int PROV>
__global__ __launch_bounds__(512) void wgrad_cl_kernel(WgradClArgs a)
{
    const int lane = threadIdx.x & 63;
    const int t = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform
    const int h = lane >> 5, c = lane & 31;
    const int b = 32 * t + c;
    const bool bok = b < a.Mb;
    // Lanes whose channel does not exist read the last channel instead: their rows/columns of
    // the accumulator are never stored, so the loads need no predicate.
    const int bl = bok ? b : a.Mb - 1;
    float vk0 = 0.f, vk1 = 0.f, vk2 = 0.f;
    if (PROV != PRO_NONE) {
        vk0 = a.vc0[bl];
        vk1 = a.vc1[bl];
        if (PROV == PRO_BNBWD)
            vk2 = a.vc2[bl];
    }
    float uk0[MTA], uk1[MTA], uk2[MTA];
    int al[MTA];
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta) {
        const int ai = 32 * ta + c;
        al[ta] = ai < a.Ma ? ai : a.Ma - 1;
        uk0[ta] = uk1[ta] = uk2[ta] = 0.f;
        if (PROU != PRO_NONE) {
            uk0[ta] = a.uc0[al[ta]];
            uk1[ta] = a.uc1[al[ta]];
            if (PROU == PRO_BNBWD)
                uk2[ta] = a.uc2[al[ta]];
        }
    }
    float16v acc[MTA];
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta)
        acc[ta] = (float16v){0};

    const int cBeg = blockIdx.x * a.chunksPerWg;
    const int cEnd = (cBeg + a.chunksPerWg < a.numChunks) ? cBeg + a.chunksPerWg : a.numChunks;
    // chunks whose 32 pixels all exist take the branch-free path, two at a time so that the
    // loads of one are in flight while the other is multiplied
    const int cFull = (int)(a.Q / 32u) < cEnd ? (int)(a.Q / 32u) : cEnd;

    auto load_chunk = [&](int ch, float (&vv)[4][4], float (&uu)[MTA][4][4]) {
        const uint32_t q0 = (uint32_t)ch * 32u + 4u * h;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const uint32_t q = q0 + 8 * jj;
            load_chan4<T, PROV>(a.v0, a.v1, a.vgate, a.Mb, a.HW, a.divHW, q, bl, vk0, vk1, vk2,
                                vv[jj]);
#pragma unroll
            for (int ta = 0; ta < MTA; ++ta)
                load_chan4<T, PROU>(a.u0, a.u1, a.ugate, a.Ma, a.HW, a.divHW, q, al[ta], uk0[ta],
                                    uk1[ta], uk2[ta], uu[ta][jj]);
        }
    };
    auto mma_chunk = [&](const float (&vv)[4][4], const float (&uu)[MTA][4][4]) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int ta = 0; ta < MTA; ++ta)
                    acc[ta] = __builtin_amdgcn_mfma_f32_32x32x2f32(uu[ta][jj][r], vv[jj][r], acc[ta],
                                                                   0, 0, 0);
    };

    int ch = cBeg;
    if (ch < cFull) {
        float vA[4][4], uA[MTA][4][4], vB[4][4], uB[MTA][4][4];
        load_chunk(ch, vA, uA);
        for (; ch + 1 < cFull; ch += 2) {
            load_chunk(ch + 1, vB, uB);
            mma_chunk(vA, uA);
            if (ch + 2 < cFull)
                load_chunk(ch + 2, vA, uA);
            mma_chunk(vB, uB);
        }
        if (ch < cFull) { // odd count: the last full chunk is already loaded in A
            mma_chunk(vA, uA);
            ++ch;
        }
    }
    for (; ch < cEnd; ++ch) { // ragged last chunk: pixels past the end contribute zero
        const uint32_t q0 = (uint32_t)ch * 32u;
        float vv[4][4], uu[MTA][4][4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const uint32_t q = q0 + 8 * jj + 4 * h;
            const bool qok = q < a.Q;
            const uint32_t qs = qok ? q : 0u;
            load_chan4<T, PROV>(a.v0, a.v1, a.vgate, a.Mb, a.HW, a.divHW, qs, bl, vk0, vk1, vk2,
                                vv[jj]);
#pragma unroll
            for (int ta = 0; ta < MTA; ++ta) {
                load_chan4<T, PROU>(a.u0, a.u1, a.ugate, a.Ma, a.HW, a.divHW, qs, al[ta], uk0[ta],
                                    uk1[ta], uk2[ta], uu[ta][jj]);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    uu[ta][jj][r] = qok ? uu[ta][jj][r] : 0.f;
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r)
                vv[jj][r] = qok ? vv[jj][r] : 0.f;
        }
        mma_chunk(vv, uu);
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

// ---- wgrad_lt: coalesced loads + LDS transpose -------------------------------------------------
// Loading operands directly in channel-lane form makes every load instruction touch 32
// different cache lines (one per channel row, 32 bytes of each), and on this chip the number of
// distinct lines per instruction, not the byte count, bounds such a kernel.  wgrad_lt loads
// 32-channel x 32-pixel operand tiles row-wise instead (8 lanes x 16 bytes per row, 8 lines per
// instruction), applies the prologue, parks the tile in LDS and reads it back channel-lane for
// the MFMA.  The narrow operand U is staged once per workgroup and shared by all wavefronts;
// each wavefront stages its own 32 channels of the wide operand V.  Global loads of chunk i+1
// are issued before the MFMAs of chunk i.

constexpr int kLtPitch = 36; // floats per LDS tile row: 16-byte aligned, conflict-free b128 reads

template <typename T, int PRO>
__device__ __forceinline__ void lt_prologue(float (&v)[4], const float (&raw)[4], float k0, float k1,
                                            float k2, float g)
{
    if (PRO == PRO_BNBWD) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            v[r] = fmaf(k0, v[r], fmaf(k1, raw[r], k2));
    } else if (PRO == PRO_BNSWISH_GATE) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            v[r] = actf(fmaf(v[r], k0, k1)) * g;
    }
}

template <typename T, int MTA, int PROU, int PROV>
__global__ __launch_bounds__(512) void wgrad_lt_kernel(WgradClArgs a)
{
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63;
    const int t = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform
    const int h = lane >> 5, c = lane & 31;
    float *Us = lds;                                             // [2][32*MTA][pitch]
    float *Vs = lds + 2 * 32 * MTA * kLtPitch + t * 32 * kLtPitch; // this wave's [32][pitch]

    // V tile, row-wise: this lane loads pixels [vcol, vcol+4) of rows lane/8 + 8i, i = 0..3
    const int vcol = 4 * (lane & 7);
    int vch[4];
    float vk0[4], vk1[4], vk2[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int ch = 32 * t + (lane >> 3) + 8 * i;
        vch[i] = ch < a.Mb ? ch : a.Mb - 1; // rows past the end are computed but never stored
        vk0[i] = vk1[i] = vk2[i] = 0.f;
        if (PROV != PRO_NONE) {
            vk0[i] = a.vc0[vch[i]];
            vk1[i] = a.vc1[vch[i]];
            if (PROV == PRO_BNBWD)
                vk2[i] = a.vc2[vch[i]];
        }
    }
    // U tile, row-wise, by the first 256 threads: row = tid/8 (+32 per extra tile), same columns
    const bool ustager = threadIdx.x < 256;
    const int urow = (threadIdx.x >> 3) & 31;
    int uch[MTA];
    float uk0[MTA], uk1[MTA], uk2[MTA];
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta) {
        const int ch = 32 * ta + urow;
        uch[ta] = ch < a.Ma ? ch : a.Ma - 1;
        uk0[ta] = uk1[ta] = uk2[ta] = 0.f;
        if (PROU != PRO_NONE) {
            uk0[ta] = a.uc0[uch[ta]];
            uk1[ta] = a.uc1[uch[ta]];
            if (PROU == PRO_BNBWD)
                uk2[ta] = a.uc2[uch[ta]];
        }
    }

    float16v acc[MTA];
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta)
        acc[ta] = (float16v){0};

    const int cBeg = blockIdx.x * a.chunksPerWg;
    const int cEnd = (cBeg + a.chunksPerWg < a.numChunks) ? cBeg + a.chunksPerWg : a.numChunks;

    float vv[4][4], vr[4][4], vg[4], uu[MTA][4], ur[MTA][4], ug[MTA];
    bool pok = true; // this lane's four pixels exist (false only in a ragged last chunk)
    auto fetch = [&](int ch) {
        const uint32_t q = (uint32_t)ch * 32u + (uint32_t)vcol;
        pok = q < a.Q;
        const uint32_t qs = pok ? q : 0u;
        const uint32_t n = fdiv(qs, a.divHW);
        const uint32_t pix = qs - n * (uint32_t)a.HW;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const size_t idx = ((size_t)n * a.Mb + vch[i]) * a.HW + pix;
            load4<T>((const T *)a.v0, idx, vv[i]);
            if (PROV == PRO_BNBWD)
                load4<T>((const T *)a.v1, idx, vr[i]);
            if (PROV == PRO_BNSWISH_GATE)
                vg[i] = a.vgate[(size_t)n * a.Mb + vch[i]];
        }
        if (ustager) {
#pragma unroll
            for (int ta = 0; ta < MTA; ++ta) {
                const size_t idx = ((size_t)n * a.Ma + uch[ta]) * a.HW + pix;
                load4<T>((const T *)a.u0, idx, uu[ta]);
                if (PROU == PRO_BNBWD)
                    load4<T>((const T *)a.u1, idx, ur[ta]);
                if (PROU == PRO_BNSWISH_GATE)
                    ug[ta] = a.ugate[(size_t)n * a.Ma + uch[ta]];
            }
        }
    };

    if (cBeg < cEnd)
        fetch(cBeg);
    for (int ch = cBeg; ch < cEnd; ++ch) {
        float *Ub = Us + ((ch - cBeg) & 1) * (32 * MTA * kLtPitch);
        // finish the prologue on the fetched registers and park the tiles in LDS
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            lt_prologue<T, PROV>(vv[i], vr[i], vk0[i], vk1[i], vk2[i], vg[i]);
            float4v w4 = {vv[i][0], vv[i][1], vv[i][2], vv[i][3]};
            if (!pok)
                w4 = (float4v){0.f, 0.f, 0.f, 0.f};
            *reinterpret_cast<float4v *>(Vs + ((lane >> 3) + 8 * i) * kLtPitch + vcol) = w4;
        }
        if (ustager) {
#pragma unroll
            for (int ta = 0; ta < MTA; ++ta) {
                lt_prologue<T, PROU>(uu[ta], ur[ta], uk0[ta], uk1[ta], uk2[ta], ug[ta]);
                float4v w4 = {uu[ta][0], uu[ta][1], uu[ta][2], uu[ta][3]};
                if (!pok)
                    w4 = (float4v){0.f, 0.f, 0.f, 0.f};
                *reinterpret_cast<float4v *>(Ub + (32 * ta + urow) * kLtPitch + vcol) = w4;
            }
        }
        __syncthreads();
        if (ch + 1 < cEnd)
            fetch(ch + 1); // in flight while this chunk is multiplied
        // channel-lane reads: lane (c, h) takes pixels 8*jj + 4*h + {0..3} of its channel row
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const float4v bvv = *reinterpret_cast<const float4v *>(Vs + c * kLtPitch + 8 * jj + 4 * h);
#pragma unroll
            for (int ta = 0; ta < MTA; ++ta) {
                const float4v avv =
                    *reinterpret_cast<const float4v *>(Ub + (32 * ta + c) * kLtPitch + 8 * jj + 4 * h);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[ta] = __builtin_amdgcn_mfma_f32_32x32x2f32(avv[r], bvv[r], acc[ta], 0, 0, 0);
            }
        }
    }
    const int b = 32 * t + c;
    float *dst = a.partial + (size_t)blockIdx.x * a.Ma * a.Mb;
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int ai = 32 * ta + 8 * (q >> 2) + 4 * h + (q & 3);
            if (ai < a.Ma && b < a.Mb)
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
        const size_t lds = sizeof(float) * kLtPitch * 32 * (2 * MTA + block.x / 64);              \
        hipLaunchKernelGGL((wgrad_lt_kernel<T, MTA, PU, PV>), grid, block, lds, st, a);           \
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
    dim3 grid((unsigned)splits), block((unsigned)(64 * (mtb < 4 ? 4 : mtb))); // >= 256 threads stage U
    return bf16 ? wgrad_cl_dispatch<bf16_t>(a, mta, u.pro, v.pro, grid, block, st)
                : wgrad_cl_dispatch<float>(a, mta, u.pro, v.pro, grid, block, st);
}

} // namespace mbk
