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
#include <type_traits>

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

template <typename T>
__device__ __forceinline__ void store4(T *p, size_t i, const float (&v)[4]);
template <>
__device__ __forceinline__ void store4<float>(float *p, size_t i, const float (&v)[4])
{
    *reinterpret_cast<float4v *>(p + i) = (float4v){v[0], v[1], v[2], v[3]};
}
template <>
__device__ __forceinline__ void store4<bf16_t>(bf16_t *p, size_t i, const float (&v)[4])
{
    uint2 t;
    t.x = bf16_pack2(v[0], v[1]);
    t.y = bf16_pack2(v[2], v[3]);
    *reinterpret_cast<uint2 *>(&p[i]) = t;
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
    // wgrad_lt with its data-gradient option (narrow -> wide convolution, U = gradient at the
    // narrow output, V = the convolution's wide input): dgw[a*Mb + b] are the weights, the
    // gradient with respect to V's tensor, sum_a dgw[a][b] * U[a][pix], goes to dgout [N,Mb,HW]
    const void *dgw;
    void *dgout;
    int dgtiles[8]; // bit tt of dgtiles[t]: wavefront t computes the data gradient of wide tile tt
    BnBwdFin ufin;  // ufin.psb non-null: U's BN-backward coefficients are derived in the kernel
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

// DG (the projection conv's backward in one kernel): the same pass also produces the gradient
// with respect to the wide operand's tensor, G[b][pix] = sum_a W[a][b] * U[a][pix].  A 32-channel
// tile of G needs only W^T (an LDS table in MFMA operand order, A) and the parked U tile read
// pixel-lane (B), so any wavefront can compute any tile and nothing is added across wavefronts.
// The tiles are dealt out by the host so that the four SIMDs, which the wavefronts of a
// workgroup occupy in turn, get equal MFMA counts (with five wavefronts the SIMD that hosts two of
// them would otherwise carry twice the load of the others and set the pace).  The 32x32 result is
// turned row-wise through the wavefront's own V tile (which its weight-gradient reads have left
// by then: LDS operations of a wavefront execute in order, no barrier) and stored 16 bytes per lane.
template <typename T, int MTA, int PROU, int PROV, bool DG>
__global__ __launch_bounds__(512, DG ? 4 : 1) void wgrad_lt_kernel(WgradClArgs a)
{
    static_assert(!DG || MTA == 1, "the data-gradient option takes one narrow tile");
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63;
    const int t = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform
    const int h = lane >> 5, c = lane & 31;
    float *Us = lds;                                             // [2][32*MTA][pitch]
    float *Vs = lds + 2 * 32 * MTA * kLtPitch + t * 32 * kLtPitch; // this wave's [32][pitch]
    // DG: [tile][16 steps][64 lanes] of W^T, behind all the tiles; each wave fills its own tile's
    float *WlAll = lds + (2 * 32 * MTA + 32 * (blockDim.x >> 6)) * kLtPitch;
    float *Wl = WlAll + t * 16 * 64;

    // V tile, row-wise: this lane loads pixels [vcol, vcol+4) of rows lane/8 + 8i, i = 0..3
    const int vcol = 4 * (lane & 7);
    int vch[4];
    uint32_t vro[4]; // element offset of the row within an image (32 bits)
    float vk0[4], vk1[4], vk2[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int ch = 32 * t + (lane >> 3) + 8 * i;
        vch[i] = ch < a.Mb ? ch : a.Mb - 1; // rows past the end are computed but never stored
        vro[i] = (uint32_t)vch[i] * (uint32_t)a.HW;
        vk0[i] = vk1[i] = vk2[i] = 0.f;
        if (PROV != PRO_NONE) {
            vk0[i] = a.vc0[vch[i]];
            vk1[i] = a.vc1[vch[i]];
            if (PROV == PRO_BNBWD)
                vk2[i] = a.vc2[vch[i]];
        }
    }
    const uint32_t vimg = (uint32_t)a.Mb * (uint32_t)a.HW, uimg = (uint32_t)a.Ma * (uint32_t)a.HW;
    // U tile, row-wise, by the first 256 threads: row = tid/8 (+32 per extra tile), same columns
    const bool ustager = threadIdx.x < 256;
    const int urow = (threadIdx.x >> 3) & 31;
    int uch[MTA];
    uint32_t uro[MTA];
    float uk0[MTA], uk1[MTA], uk2[MTA];
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta) {
        const int ch = 32 * ta + urow;
        uch[ta] = ch < a.Ma ? ch : a.Ma - 1;
        uro[ta] = (uint32_t)uch[ta] * (uint32_t)a.HW;
        uk0[ta] = uk1[ta] = uk2[ta] = 0.f;
        if (DG && PROU == PRO_BNBWD && a.ufin.psb) {
            // The normalisation's backward finalise step, here instead of in a launch of its own:
            // the eight lanes that stage a row of U add that channel's partial sums (lane s takes
            // partials s, s+8, ...; fp64; a fixed butterfly over the eight), every workgroup in
            // the same order, so all arrive at the same coefficients; workgroup 0 stores them.
            if (ustager) { // whole wavefronts
                const int ch = uch[ta], sub = threadIdx.x & 7, NP = a.ufin.NP, Cn = a.Ma;
                const float gm = a.ufin.gamma[ch], mean = a.ufin.bn[2 * Cn + ch];
                const float rstd = a.ufin.bn[3 * Cn + ch];
                const float *pb = a.ufin.psb + (size_t)ch * NP, *pr = a.ufin.psr + (size_t)ch * NP;
                double sb = 0.0, sr = 0.0;
                for (int i0 = sub; i0 < NP; i0 += 32) {
                    float b0[4], b1[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int i = min(i0 + 8 * u, NP - 1); // unconditional loads, masked below
                        b0[u] = pb[i];
                        b1[u] = pr[i];
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (i0 + 8 * u < NP) {
                            sb += (double)b0[u];
                            sr += (double)b1[u];
                        }
                }
#pragma unroll
                for (int o = 4; o > 0; o >>= 1) {
                    sb += __shfl_xor(sb, o, kWave);
                    sr += __shfl_xor(sr, o, kWave);
                }
                // c0*dy + c1*raw + c2 (see launch_bn_bwd_finalize): dgamma = sr, dbeta = sb
                const double c0 = (double)gm * rstd;
                const double c1 = -c0 * rstd * sr / a.ufin.m;
                const double c2 = -c0 * sb / a.ufin.m - c1 * mean;
                uk0[ta] = (float)c0;
                uk1[ta] = (float)c1;
                uk2[ta] = (float)c2;
                if (blockIdx.x == 0 && sub == 0 && 32 * ta + urow < Cn) {
                    a.ufin.dbeta[ch] = (float)sb;
                    a.ufin.dgamma[ch] = (float)sr;
                    a.ufin.coef[ch] = uk0[ta];
                    a.ufin.coef[Cn + ch] = uk1[ta];
                    a.ufin.coef[2 * Cn + ch] = uk2[ta];
                }
            }
        } else if (PROU != PRO_NONE) {
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

    // Chunks are dealt out round-robin: at any moment the workgroups in flight read neighbouring
    // 128-byte pieces of every channel row instead of pieces chunksPerWg*128 bytes apart.
    const int cBeg = blockIdx.x, cStep = gridDim.x, cEnd = a.numChunks;

    if (DG) {
        // lane (h, c), step kk holds W[a = 2kk + h][b = 32t + c], zero outside the matrix; all
        // sixteen loads issued before the first store
        float wreg[16];
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const int aa = 2 * kk + h, bb = 32 * t + c;
            const bool ok = aa < a.Ma && bb < a.Mb;
            wreg[kk] = and_mask(ld<T>((const T *)a.dgw, ok ? (size_t)aa * a.Mb + bb : 0),
                                ok ? 0xffffffffu : 0u);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < 16; ++kk)
            Wl[kk * 64 + lane] = wreg[kk]; // first read after the first chunk's barrier
    }
    const int kdg = (a.Ma + 1) >> 1; // contraction steps of the data gradient
    const int dgmask = DG ? a.dgtiles[t] : 0; // wave-uniform

    float vv[4][4], vr[4][4], vg[4], uu[MTA][4], ur[MTA][4], ug[MTA];
    size_t vbase_cur = 0; // DG: where this lane's rows of the current chunk start
    bool pok = true; // this lane's four pixels exist (false only in a ragged last chunk)
    auto fetch = [&](int ch) {
        const uint32_t q = (uint32_t)ch * 32u + (uint32_t)vcol;
        pok = q < a.Q;
        const uint32_t qs = pok ? q : 0u;
        const uint32_t n = fdiv(qs, a.divHW);
        const uint32_t pix = qs - n * (uint32_t)a.HW;
        // (one 64-bit multiply-add per chunk and an addition per load)
        const size_t vbase = (size_t)n * vimg + pix;
        vbase_cur = vbase;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const size_t idx = vbase + vro[i];
            load4<T>((const T *)a.v0, idx, vv[i]);
            if (PROV == PRO_BNBWD)
                load4<T>((const T *)a.v1, idx, vr[i]);
            if (PROV == PRO_BNSWISH_GATE)
                vg[i] = a.vgate[(size_t)n * a.Mb + vch[i]];
        }
        if (ustager) {
            const size_t ubase = (size_t)n * uimg + pix;
#pragma unroll
            for (int ta = 0; ta < MTA; ++ta) {
                const size_t idx = ubase + uro[ta];
                load4<T>((const T *)a.u0, idx, uu[ta]);
                if (PROU == PRO_BNBWD)
                    load4<T>((const T *)a.u1, idx, ur[ta]);
                if (PROU == PRO_BNSWISH_GATE)
                    ug[ta] = a.ugate[(size_t)n * a.Ma + uch[ta]];
            }
        }
    };

    // One chunk.  `more` (a compile-time flag: the last chunk gets a copy of the body without the
    // loads, so that every wait in both copies counts a fixed number of outstanding loads) says
    // whether another chunk follows; its operands are requested as soon as this chunk's have been
    // parked, before the barrier.
    const auto body = [&](int ch, int it, auto more) {
        float *Ub = Us + (it & 1) * (32 * MTA * kLtPitch);
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
        const size_t gbase = vbase_cur;
        const bool gok = pok;
        if (decltype(more)::value)
            fetch(ch + cStep); // in flight while this chunk is multiplied
        __syncthreads();
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
        if (DG) {
            for (int tt = 0; (dgmask >> tt) != 0; ++tt) {
                if (!((dgmask >> tt) & 1))
                    continue;
                const float *Wt = WlAll + tt * 16 * 64;
                // pixel-lane reads of the U tile: lane (h, c) takes U[2kk + h][pixel c]
                float16v accd = (float16v){0};
                int kk = 0;
                for (; kk + 4 <= kdg; kk += 4) {
                    float dv[4], wv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        dv[u] = Ub[(2 * (kk + u) + h) * kLtPitch + c];
                        wv[u] = Wt[(kk + u) * 64 + lane];
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        accd = __builtin_amdgcn_mfma_f32_32x32x2f32(wv[u], dv[u], accd, 0, 0, 0);
                }
                for (; kk < kdg; ++kk)
                    accd = __builtin_amdgcn_mfma_f32_32x32x2f32(Wt[kk * 64 + lane],
                                                                Ub[(2 * kk + h) * kLtPitch + c], accd, 0, 0, 0);
                // accumulator register q holds channel row 8*(q/4) + 4h + q%4, pixel c
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    Vs[(8 * (q >> 2) + 4 * h + (q & 3)) * kLtPitch + c] = accd[q];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = (lane >> 3) + 8 * i, ch = 32 * tt + row;
                    const float4v g4 = *reinterpret_cast<const float4v *>(Vs + row * kLtPitch + vcol);
                    if (gok && ch < a.Mb) {
                        const float o[4] = {g4[0], g4[1], g4[2], g4[3]};
                        store4<T>((T *)a.dgout, gbase + (uint32_t)ch * (uint32_t)a.HW, o);
                    }
                }
            }
        }
    };
    if (cBeg < cEnd) {
        fetch(cBeg);
        int it = 0, ch = cBeg;
        for (; ch + cStep < cEnd; ch += cStep, ++it)
            body(ch, it, std::true_type{});
        body(ch, it, std::false_type{});
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

// Arguments of the expansion conv's fused backward kernel (bwd1x1_lt).
struct Bwd1x1Args {
    WgradClArgs g; // U = x (PRO_NONE), V = de (PRO_BNBWD); partial: weight-gradient splits
    int kbeg[9];   // wavefront t multiplies contraction steps [kbeg[t], kbeg[t+1]) of the data gradient
    const void *w; // [Mb][Ma] in the activation dtype (wide-major, as the layer stores it)
    void *dx;      // [N][Ma][HW]
    const void *res; // optional, added to dx
};

// ---- wave-per-chunk form of the projection conv's fused backward ---------------------------------
// In wgrad_lt<..., DG> a workgroup shares one 32-pixel chunk: every wavefront
// stages 32 wide channels of it and two workgroup barriers per chunk hold all of them to the
// pace of the slowest (with at most 32 wide channels, the block without an expansion conv, one
// wavefront did all the work while the others waited).  Here every wavefront is on its own: it
// takes 32-pixel chunks round-robin and walks the NTW 32-channel tiles of the wide side itself,
// with LDS tiles of its own, so the pixel loop has no workgroup barrier at all (a wavefront's
// LDS operations execute in order; a wave-scope fence keeps the compiler from reordering them).
// The next tile's (and the next chunk's) operands are requested before the current tile is
// multiplied.  What is constant over the loop (W in MFMA operand order, BN coefficients) waits
// in LDS tables shared by the workgroup.  The four wavefronts' weight-gradient tiles are added
// in wavefront order at the end and the workgroups' partial tiles by reduce_splits: fixed
// order, no atomics.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Adds the four wavefronts' NTW accumulator tiles (rows = narrow channels, columns = wide) in
// wavefront order, one tile at a time through 16 KB of LDS, and stores them to `dst`.
template <int NTW>
__device__ __forceinline__ void wave_tiles_reduce_store(const float16v (&acc)[NTW], float *Rd, int t,
                                                        int lane, int Ma, int Mb, int sOa, int sOb,
                                                        float *dst)
{
#pragma unroll
    for (int tt = 0; tt < NTW; ++tt) {
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 16; ++q)
            Rd[(t * 16 + q) * 64 + lane] = acc[tt][q];
        __syncthreads();
        for (int e = threadIdx.x; e < 16 * 64; e += 256) {
            const int q = e >> 6, l = e & 63;
            const float s = (Rd[e] + Rd[1024 + e]) + (Rd[2048 + e] + Rd[3072 + e]);
            const int ai = 8 * (q >> 2) + 4 * (l >> 5) + (q & 3), bi = 32 * tt + (l & 31);
            if (ai < Ma && bi < Mb)
                dst[(size_t)ai * sOa + (size_t)bi * sOb] = s;
        }
    }
}

// Projection conv backward, Cn <= 32 narrow output channels, Cw <= 32*NTW wide input channels:
// U = dp (BN3's backward of dout and p, coefficients finalised here from the partial sums as in
// wgrad_lt<..., DG>), V = sc = act(BN2(d))*gate.  Per chunk and wide tile: the weight gradient
// dW[a][b] += sum_pix dp[a][pix]*sc[b][pix] (16 MFMAs, both tiles read channel-lane) and the data
// gradient G[b][pix] = sum_a W[a][b]*dp[a][pix] (ceil(Cn/2) MFMAs, W^T from the LDS table, the U
// tile read pixel-lane), turned row-wise through the V tile and stored 16 bytes per lane.
template <typename T, int PROV, int NTW>
__global__ __launch_bounds__(256, NTW == 1 ? 3 : 2) void projbwd_wave_kernel(WgradClArgs a)
{
    extern __shared__ float lds[];
    constexpr int R = 32 * NTW;
    const int lane = threadIdx.x & 63;
    const int t = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform
    const int h = lane >> 5, c = lane & 31;
    float *Ut = lds + t * (2 * 32 * kLtPitch); // this wavefront's [32][pitch]
    float *Vt = Ut + 32 * kLtPitch;            // this wavefront's [32][pitch]
    float *Cl = lds + 4 * (2 * 32 * kLtPitch); // [3][32]: c0, c1, c2 of U's rows
    float *Cv = Cl + 96;                       // [2][R]: scale and shift of V's rows
    float *Wl = Cv + 2 * R;                    // [NTW][16 steps][64 lanes] of W^T in MFMA operand order

    // ---- BN3 backward coefficients of the (at most 32) rows of U: thread (row = tid/8, sub = tid%8)
    {
        const int row = threadIdx.x >> 3, sub = threadIdx.x & 7, Cn = a.Ma;
        const int ch = row < Cn ? row : Cn - 1;
        float k0, k1, k2;
        if (a.ufin.psb) {
            const int NP = a.ufin.NP;
            const float gm = a.ufin.gamma[ch], mean = a.ufin.bn[2 * Cn + ch];
            const float rstd = a.ufin.bn[3 * Cn + ch];
            const float *pb = a.ufin.psb + (size_t)ch * NP, *pr = a.ufin.psr + (size_t)ch * NP;
            double sb = 0.0, sr = 0.0;
            for (int i0 = sub; i0 < NP; i0 += 32) {
                float b0[4], b1[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = min(i0 + 8 * u, NP - 1); // unconditional loads, masked below
                    b0[u] = pb[i];
                    b1[u] = pr[i];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (i0 + 8 * u < NP) {
                        sb += (double)b0[u];
                        sr += (double)b1[u];
                    }
            }
#pragma unroll
            for (int o = 4; o > 0; o >>= 1) {
                sb += __shfl_xor(sb, o, kWave);
                sr += __shfl_xor(sr, o, kWave);
            }
            // c0*dy + c1*raw + c2 (see launch_bn_bwd_finalize): dgamma = sr, dbeta = sb
            const double c0 = (double)gm * rstd;
            const double c1 = -c0 * rstd * sr / a.ufin.m;
            const double c2 = -c0 * sb / a.ufin.m - c1 * mean;
            k0 = (float)c0;
            k1 = (float)c1;
            k2 = (float)c2;
            if (blockIdx.x == 0 && sub == 0 && row < Cn) {
                a.ufin.dbeta[ch] = (float)sb;
                a.ufin.dgamma[ch] = (float)sr;
                a.ufin.coef[ch] = k0;
                a.ufin.coef[Cn + ch] = k1;
                a.ufin.coef[2 * Cn + ch] = k2;
            }
        } else {
            k0 = a.uc0[ch];
            k1 = a.uc1[ch];
            k2 = a.uc2[ch];
        }
        if (sub == 0) { // rows past the end of U must contribute zero to both products
            Cl[row] = row < Cn ? k0 : 0.f;
            Cl[32 + row] = row < Cn ? k1 : 0.f;
            Cl[64 + row] = row < Cn ? k2 : 0.f;
        }
    }
    // W^T as the data gradient's A operand: lane (h, c), tile tt, step kk holds
    // W[a = 2kk + h][b = 32tt + c]; 4*NTW entries per thread, loads before stores
    {
        float wreg[4 * NTW];
#pragma unroll
        for (int i = 0; i < 4 * NTW; ++i) {
            const int e = threadIdx.x + 256 * i, l = e & 63, kk = (e >> 6) & 15, tt = e >> 10;
            const int aa = 2 * kk + (l >> 5), bb = 32 * tt + (l & 31);
            const bool ok = aa < a.Ma && bb < a.Mb;
            wreg[i] = and_mask(ld<T>((const T *)a.dgw, ok ? (size_t)aa * a.Mb + bb : 0), ok ? 0xffffffffu : 0u);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4 * NTW; ++i)
            Wl[threadIdx.x + 256 * i] = wreg[i];
        for (int r = threadIdx.x; r < R; r += 256) {
            const int ch = r < a.Mb ? r : a.Mb - 1;
            Cv[r] = PROV != PRO_NONE ? a.vc0[ch] : 0.f;
            Cv[R + r] = PROV != PRO_NONE ? a.vc1[ch] : 0.f;
        }
    }
    // rows this lane stages: lane/8 + 8i of a tile, pixels [vcol, vcol+4) of the chunk
    const int vcol = 4 * (lane & 7), lrow = lane >> 3;
    uint32_t uro[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = lrow + 8 * i;
        uro[i] = (uint32_t)(row < a.Ma ? row : a.Ma - 1) * (uint32_t)a.HW;
    }
    __syncthreads(); // Cl, Cv, Wl
    const uint32_t vimg = (uint32_t)a.Mb * (uint32_t)a.HW, uimg = (uint32_t)a.Ma * (uint32_t)a.HW;
    const int kdg = (a.Ma + 1) >> 1;

    float16v acc[NTW];
#pragma unroll
    for (int tt = 0; tt < NTW; ++tt)
        acc[tt] = (float16v){0};
    float vv[4][4], vg[4], uu[4][4], ur[4][4];
    struct Geom {
        uint32_t n, pix;
        bool ok; // this lane's four pixels exist (false only in a ragged last chunk)
    };
    auto geom = [&](int ch) {
        Geom g;
        const uint32_t q = (uint32_t)ch * 32u + (uint32_t)vcol;
        g.ok = q < a.Q;
        const uint32_t qs = g.ok ? q : 0u;
        g.n = fdiv(qs, a.divHW);
        g.pix = qs - g.n * (uint32_t)a.HW;
        return g;
    };
    auto fetchU = [&](const Geom &g) {
        const size_t ubase = (size_t)g.n * uimg + g.pix;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            load4<T>((const T *)a.u0, ubase + uro[i], uu[i]);
            load4<T>((const T *)a.u1, ubase + uro[i], ur[i]);
        }
    };
    auto fetchV = [&](const Geom &g, int tt) {
        const size_t vbase = (size_t)g.n * vimg + g.pix;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 32 * tt + lrow + 8 * i;
            const int ch = row < a.Mb ? row : a.Mb - 1; // rows past the end are computed but never stored
            load4<T>((const T *)a.v0, vbase + (uint32_t)ch * (uint32_t)a.HW, vv[i]);
            if (PROV == PRO_BNSWISH_GATE)
                vg[i] = a.vgate[(size_t)g.n * a.Mb + ch];
        }
    };
    const auto body = [&](const Geom &g, const Geom &gn, auto more) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = lrow + 8 * i;
            lt_prologue<T, PRO_BNBWD>(uu[i], ur[i], Cl[row], Cl[32 + row], Cl[64 + row], 0.f);
            float4v u4 = {uu[i][0], uu[i][1], uu[i][2], uu[i][3]};
            if (!g.ok)
                u4 = (float4v){0.f, 0.f, 0.f, 0.f};
            *reinterpret_cast<float4v *>(Ut + row * kLtPitch + vcol) = u4;
        }
        if (decltype(more)::value)
            fetchU(gn); // the next chunk's U tile: in flight while this chunk is multiplied
        const size_t gbase = (size_t)g.n * vimg + g.pix;
#pragma unroll
        for (int tt = 0; tt < NTW; ++tt) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = lrow + 8 * i;
                lt_prologue<T, PROV>(vv[i], vv[i], Cv[32 * tt + row], Cv[R + 32 * tt + row], 0.f, vg[i]);
                float4v v4 = {vv[i][0], vv[i][1], vv[i][2], vv[i][3]};
                if (!g.ok)
                    v4 = (float4v){0.f, 0.f, 0.f, 0.f};
                *reinterpret_cast<float4v *>(Vt + row * kLtPitch + vcol) = v4;
            }
            if (tt + 1 < NTW)
                fetchV(g, tt + 1); // in flight while this tile is multiplied
            else if (decltype(more)::value)
                fetchV(gn, 0);
            wave_lds_fence();
            // weight gradient, channel-lane reads: lane (c, h) takes pixels 8*jj + 4*h + {0..3} of row c
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const float4v bvv = *reinterpret_cast<const float4v *>(Vt + c * kLtPitch + 8 * jj + 4 * h);
                const float4v avv = *reinterpret_cast<const float4v *>(Ut + c * kLtPitch + 8 * jj + 4 * h);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[tt] = __builtin_amdgcn_mfma_f32_32x32x2f32(avv[r], bvv[r], acc[tt], 0, 0, 0);
            }
            // data gradient, pixel-lane reads of the U tile: lane (h, c) takes U[2kk + h][pixel c]
            float16v accd = (float16v){0};
#pragma unroll
            for (int k4 = 0; k4 < 16; k4 += 4) {
                if (k4 < kdg) { // wave-uniform
                    float dv[4], wv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        dv[u] = Ut[(2 * (k4 + u) + h) * kLtPitch + c];
                        wv[u] = Wl[(tt * 16 + k4 + u) * 64 + lane];
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        accd = __builtin_amdgcn_mfma_f32_32x32x2f32(wv[u], dv[u], accd, 0, 0, 0);
                }
            }
            // accumulator register q holds channel row 8*(q/4) + 4h + q%4, pixel c: through the V
            // tile (its reads are behind us: LDS operations of a wavefront execute in order)
#pragma unroll
            for (int q = 0; q < 16; ++q)
                Vt[(8 * (q >> 2) + 4 * h + (q & 3)) * kLtPitch + c] = accd[q];
            wave_lds_fence();
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = lrow + 8 * i, ch = 32 * tt + row;
                const float4v g4 = *reinterpret_cast<const float4v *>(Vt + row * kLtPitch + vcol);
                if (g.ok && ch < a.Mb) {
                    const float o[4] = {g4[0], g4[1], g4[2], g4[3]};
                    store4<T>((T *)a.dgout, gbase + (uint32_t)ch * (uint32_t)a.HW, o);
                }
            }
            wave_lds_fence();
        }
    };
    const int cStep = 4 * (int)gridDim.x, cEnd = a.numChunks;
    int ch = 4 * (int)blockIdx.x + t;
    if (ch < cEnd) {
        Geom g = geom(ch);
        fetchU(g);
        fetchV(g, 0);
        for (; ch + cStep < cEnd; ch += cStep) {
            const Geom gn = geom(ch + cStep);
            body(g, gn, std::true_type{});
            g = gn;
        }
        body(g, g, std::false_type{});
    }
    wave_tiles_reduce_store<NTW>(acc, lds, t, lane, a.Ma, a.Mb, a.sOa, a.sOb,
                                 a.partial + (size_t)blockIdx.x * a.Ma * a.Mb);
}

// ---- bwd1x1_lt: data and weight gradient of a narrow->wide 1x1 convolution in one pass ---------
// The expansion conv's two gradients, dx = W^T de (+ dout) and dW = de x^T, both consume
// de = c0*dy1 + c1*e + c2 (BN1's backward applied on the fly), two wide tensors that are by far
// the largest operands; computing them in separate kernels reads both twice.  This kernel is
// wgrad_lt (U = x, the narrow input; V = de, the wide side) that also multiplies each wavefront's
// parked 32-channel x 32-pixel tile of de by its 32 rows of W:
//   P_t[j][pix] = sum_{c in wavefront t} W[c][j] * de[c][pix]     (MFMA: A = W^T from registers,
//                                                                   B = de read pixel-lane from LDS)
// (any wavefront can take any step of that contraction, the tiles being in LDS: the steps are
// dealt out so that the four SIMDs of a CU, which the wavefronts of a workgroup occupy in turn,
// get equal numbers of MFMAs although only the first ceil(Mb/32) wavefronts have weight-gradient
// work.)  The wavefronts' P_t go through LDS and are added in wavefront order by the threads that staged
// x: thread (row j, four pixels) owns exactly that element group of dx, so its address, its
// validity and the residual it adds are those of its x load.  All wide channels of a pixel live
// in one workgroup: dx needs no second stage.  Fixed summation order, no atomics.
// (Section "Guided Optimization Case Study: EfficientNet": fusing the consumers of a tensor.)


template <typename T, int MTA>
__global__ __launch_bounds__(512, 4) void bwd1x1_lt_kernel(Bwd1x1Args b)
{
    const WgradClArgs &a = b.g;
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63;
    const int t = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform
    const int nw = blockDim.x >> 6, R = 32 * nw;
    const int h = lane >> 5, c = lane & 31;
    float *Us = lds;                                               // [2][32*MTA][pitch]
    float *Vs = lds + 2 * 32 * MTA * kLtPitch + t * 32 * kLtPitch;   // this wave's [32][pitch]
    float *Pd = lds + (2 * 32 * MTA + R) * kLtPitch;                 // [nw][32*MTA][pitch]
    const float *Vall = lds + 2 * 32 * MTA * kLtPitch;               // all waves' tiles: [R][pitch]
    float *Wl = Pd + (size_t)R * MTA * kLtPitch;                     // [R/2 steps][MTA][64]
    float *Cl = Wl + (size_t)(R / 2) * MTA * 64;                     // [3][R]
    // (registers are what limits the workgroups per CU here: everything that is constant over the
    // pixel loop and not needed every cycle waits in LDS)

    // V tile (de), row-wise: this lane loads pixels [vcol, vcol+4) of rows lane/8 + 8i, i = 0..3
    const int vcol = 4 * (lane & 7);
    const int vrow = 32 * t + (lane >> 3);
    // (element offsets of this lane's rows within an image, 32 bits: the per-chunk address
    // arithmetic is one 64-bit multiply-add and an addition per load)
    uint32_t vro[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int ch = vrow + 8 * i;
        // rows past the end meet zero weights, and are never stored
        vro[i] = (uint32_t)(ch < a.Mb ? ch : a.Mb - 1) * (uint32_t)a.HW;
    }
    const uint32_t vimg = (uint32_t)a.Mb * (uint32_t)a.HW, uimg = (uint32_t)a.Ma * (uint32_t)a.HW;
    const int kb = b.kbeg[t], ke = b.kbeg[t + 1]; // wave-uniform
    // U tile (x), row-wise, by the first 256 threads: row = tid/8 (+32 per extra tile)
    const bool ustager = threadIdx.x < 256;
    const int urow = (threadIdx.x >> 3) & 31;
    uint32_t uro[MTA];
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta) {
        const int ch = 32 * ta + urow;
        uro[ta] = (uint32_t)(ch < a.Ma ? ch : a.Ma - 1) * (uint32_t)a.HW;
    }

    float16v acc[MTA];
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta)
        acc[ta] = (float16v){0};

    // Chunks are dealt out round-robin: at any moment the workgroups in flight read neighbouring
    // 128-byte pieces of every channel row (DRAM pages and cache sectors are shared between them)
    // instead of pieces chunksPerWg*128 bytes apart.
    const int cBeg = blockIdx.x, cStep = gridDim.x, cEnd = a.numChunks;

    float vv[4][4], vr[4][4], uu[MTA][4];
    size_t uidx[MTA];
    bool pok = true; // this lane's four pixels exist (false only in a ragged last chunk)
    auto fetch = [&](int ch) {
        const uint32_t q = (uint32_t)ch * 32u + (uint32_t)vcol;
        pok = q < a.Q;
        const uint32_t qs = pok ? q : 0u;
        const uint32_t n = fdiv(qs, a.divHW);
        const uint32_t pix = qs - n * (uint32_t)a.HW;
        const size_t vbase = (size_t)n * vimg + pix;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const size_t idx = vbase + vro[i];
            load4<T>((const T *)a.v0, idx, vv[i]);
            load4<T>((const T *)a.v1, idx, vr[i]);
        }
        if (ustager) {
            const size_t ubase = (size_t)n * uimg + pix;
#pragma unroll
            for (int ta = 0; ta < MTA; ++ta) {
                uidx[ta] = ubase + uro[ta];
                load4<T>((const T *)a.u0, uidx[ta], uu[ta]);
            }
        }
    };

    // BN-backward coefficients of every wide row
    for (int r = threadIdx.x; r < R; r += blockDim.x) {
        const int ch = r < a.Mb ? r : a.Mb - 1;
        Cl[r] = a.vc0[ch];
        Cl[R + r] = a.vc1[ch];
        Cl[2 * R + r] = a.vc2[ch];
    }
    // W as the data gradient's MFMA A operand: for contraction step k, lane (h, c) holds
    // W[2k + h][32ta + c]; zero outside the matrix.  (R/2)*MTA*64 entries, blockDim = 2R threads:
    // 16*MTA per thread, all loads issued before the first store (one memory round trip, not
    // sixteen).  (Measured: requesting the first chunk's operands ahead of these tables, or
    // together with them, is slower than after them.)
    {
        float wreg[16 * MTA];
#pragma unroll
        for (int i = 0; i < 16 * MTA; ++i) {
            const int e = threadIdx.x + i * (int)blockDim.x;
            const int l = e & 63, ta = (e >> 6) % MTA, k = (e >> 6) / MTA;
            const int cw = 2 * k + (l >> 5), jn = 32 * ta + (l & 31);
            const bool ok = cw < a.Mb && jn < a.Ma;
            wreg[i] = and_mask(ld<T>((const T *)b.w, ok ? (size_t)cw * a.Ma + jn : 0),
                               ok ? 0xffffffffu : 0u);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 16 * MTA; ++i)
            Wl[threadIdx.x + i * (int)blockDim.x] = wreg[i];
    }
    if (cBeg < cEnd)
        fetch(cBeg);
    __syncthreads(); // Cl, Wl
    // One chunk.  `more` (a compile-time flag: the last chunk gets a copy of the body without the
    // loads, so that every wait in both copies counts a fixed number of outstanding loads) says
    // whether another chunk follows; its operands are requested as soon as this chunk's have been
    // parked, before the barrier.
    const auto body = [&](int ch, int it, auto more) {
        float *Ub = Us + (it & 1) * (32 * MTA * kLtPitch);
        // finish the prologue on the fetched registers and park the tiles in LDS
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = vrow + 8 * i;
            lt_prologue<T, PRO_BNBWD>(vv[i], vr[i], Cl[r], Cl[R + r], Cl[2 * R + r], 0.f);
            float4v w4 = {vv[i][0], vv[i][1], vv[i][2], vv[i][3]};
            if (!pok)
                w4 = (float4v){0.f, 0.f, 0.f, 0.f};
            *reinterpret_cast<float4v *>(Vs + ((lane >> 3) + 8 * i) * kLtPitch + vcol) = w4;
        }
        // what this thread needs later to finish its element group of dx for this chunk
        size_t oidx[MTA];
        const bool ook = pok;
        if (ustager) {
#pragma unroll
            for (int ta = 0; ta < MTA; ++ta) {
                float4v w4 = {uu[ta][0], uu[ta][1], uu[ta][2], uu[ta][3]};
                if (!pok)
                    w4 = (float4v){0.f, 0.f, 0.f, 0.f};
                *reinterpret_cast<float4v *>(Ub + (32 * ta + urow) * kLtPitch + vcol) = w4;
                oidx[ta] = uidx[ta];
            }
        }
        // the residual of this chunk's dx elements, then the next chunk's operands: both in
        // flight while this chunk is multiplied
        float ores[MTA][4];
        if (ustager) {
#pragma unroll
            for (int ta = 0; ta < MTA; ++ta) {
                if (b.res) {
                    load4<T>((const T *)b.res, oidx[ta], ores[ta]);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        ores[ta][r] = 0.f;
                }
            }
        }
        if (decltype(more)::value)
            fetch(ch + cStep);
        __syncthreads();
        // weight gradient: channel-lane reads, lane (c, h) takes pixels 8*jj + 4*h + {0..3} of
        // its channel row
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
        // data gradient, this wave's share of the contraction: pixel-lane reads, lane (h, c)
        // takes de[2k+h][c]
        float16v accd[MTA];
#pragma unroll
        for (int ta = 0; ta < MTA; ++ta)
            accd[ta] = (float16v){0};
        {
            // four steps at a time: their LDS reads go out together, ahead of the four MFMAs
            int k = kb;
            for (; k + 4 <= ke; k += 4) {
                float dv[4], wv[4][MTA];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    dv[u] = Vall[(2 * (k + u) + h) * kLtPitch + c];
#pragma unroll
                    for (int ta = 0; ta < MTA; ++ta)
                        wv[u][ta] = Wl[((k + u) * MTA + ta) * 64 + lane];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int ta = 0; ta < MTA; ++ta)
                        accd[ta] = __builtin_amdgcn_mfma_f32_32x32x2f32(wv[u][ta], dv[u], accd[ta], 0, 0, 0);
            }
            for (; k < ke; ++k) {
                const float dv = Vall[(2 * k + h) * kLtPitch + c];
#pragma unroll
                for (int ta = 0; ta < MTA; ++ta)
                    accd[ta] = __builtin_amdgcn_mfma_f32_32x32x2f32(Wl[(k * MTA + ta) * 64 + lane], dv,
                                                                    accd[ta], 0, 0, 0);
            }
        }
#pragma unroll
        for (int ta = 0; ta < MTA; ++ta)
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int j = 32 * ta + 8 * (q >> 2) + 4 * h + (q & 3);
                Pd[((size_t)t * 32 * MTA + j) * kLtPitch + c] = accd[ta][q];
            }
        __syncthreads();
        if (ustager) {
#pragma unroll
            for (int ta = 0; ta < MTA; ++ta) {
                float o[4] = {ores[ta][0], ores[ta][1], ores[ta][2], ores[ta][3]};
                for (int w = 0; w < nw; ++w) {
                    const float4v pv = *reinterpret_cast<const float4v *>(
                        Pd + ((size_t)w * 32 * MTA + 32 * ta + urow) * kLtPitch + vcol);
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        o[r] += pv[r];
                }
                if (ook && 32 * ta + urow < a.Ma)
                    store4<T>((T *)b.dx, oidx[ta], o);
            }
        }
    };
    if (cBeg < cEnd) {
        int it = 0, ch = cBeg;
        for (; ch + cStep < cEnd; ch += cStep, ++it)
            body(ch, it, std::true_type{});
        body(ch, it, std::false_type{});
    }
    const int bcol = 32 * t + c;
    float *dst = a.partial + (size_t)blockIdx.x * a.Ma * a.Mb;
#pragma unroll
    for (int ta = 0; ta < MTA; ++ta)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int ai = 32 * ta + 8 * (q >> 2) + 4 * h + (q & 3);
            if (ai < a.Ma && bcol < a.Mb)
                dst[(size_t)ai * a.sOa + (size_t)bcol * a.sOb] = acc[ta][q];
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
        hipLaunchKernelGGL((wgrad_lt_kernel<T, MTA, PU, PV, false>), grid, block, lds, st, a);    \
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

bool projbwd_fused_plan(int N, int Cw, int Cn, int HW, int *splits)
{
    bool swap;
    return Cn <= 32 && Cn < Cw && wgrad_cl_plan(Cn, Cw, N, HW, &swap, splits) && !swap;
}

hipError_t launch_projbwd_fused(bool bf16, int N, int Cw, int Cn, int HW, const Operand &dp,
                                const Operand &sc, const void *w, void *G, float *partial,
                                int *splits_out, const BnBwdFin *fin, hipStream_t st)
{
    int splits;
    if (!projbwd_fused_plan(N, Cw, Cn, HW, &splits) || dp.pro != PRO_BNBWD ||
        (sc.pro != PRO_BNSWISH_GATE && sc.pro != PRO_NONE))
        return hipErrorInvalidValue;
    WgradClArgs a = {};
    a.N = N;
    a.Ma = Cn;
    a.Mb = Cw;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    a.numChunks = (int)((a.Q + 31u) / 32u);
    a.chunksPerWg = (a.numChunks + splits - 1) / splits;
    a.divHW = make_div((uint32_t)HW);
    a.u0 = dp.p0;
    a.u1 = dp.p1;
    a.uc0 = dp.c0;
    a.uc1 = dp.c1;
    a.uc2 = dp.c2;
    a.v0 = sc.p0;
    a.vc0 = sc.c0;
    a.vc1 = sc.c1;
    a.vgate = sc.gate;
    a.sOa = Cw; // dW is [Cn][Cw] row-major
    a.sOb = 1;
    a.partial = partial;
    a.dgw = w;
    a.dgout = G;
    if (fin)
        a.ufin = *fin;
    *splits_out = splits;
    const int mtb = (Cw + 31) / 32, nw = mtb < 4 ? 4 : mtb;
    const size_t lds = sizeof(float) * ((size_t)kLtPitch * 32 * (2 + nw) + (size_t)nw * 16 * 64);
    // Deal the data gradient's tiles out to the wavefronts: wavefront t runs on SIMD t % 4 and
    // already has 16 MFMAs per chunk if it owns a weight-gradient tile; a data-gradient tile is
    // ceil(Cn/2) more.  Each tile goes to the least loaded wavefront of the least loaded SIMD.
    {
        const int cost = (Cn + 1) / 2;
        int load[4] = {0, 0, 0, 0}, wload[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int t = 0; t < nw; ++t)
            if (t < mtb) {
                load[t % 4] += 16;
                wload[t] = 16;
            }
        for (int tt = 0; tt < mtb; ++tt) {
            int sbest = 0;
            for (int sd = 1; sd < 4; ++sd)
                if (load[sd] < load[sbest])
                    sbest = sd;
            int tbest = sbest;
            for (int t = sbest; t < nw; t += 4)
                if (wload[t] < wload[tbest])
                    tbest = t;
            a.dgtiles[tbest] |= 1 << tt;
            load[sbest] += cost;
            wload[tbest] += cost;
        }
    }
    dim3 grid((unsigned)splits), block((unsigned)(64 * nw));
    // wide sides of up to three tiles (96 channels): a wavefront per pixel chunk.  (Measured with
    // five and six tiles, 144 and 192 channels: the accumulator tiles of all of them plus the
    // prefetch registers no longer fit two wavefronts per SIMD without spilling, and the
    // workgroup-per-chunk kernel is faster there.  The expansion conv's fused backward in this form
    // measured no faster than bwd1x1_lt on 16 -> 96 channels, 164 against 169 us, and was dropped.)
    const int ntw = (Cw + 31) / 32;
    if (fin && ntw <= 3) {
        const size_t wv_lds = sizeof(float) * (4 * 2 * 32 * kLtPitch + 96 + 2 * 32 * ntw + (size_t)ntw * 16 * 64);
#define MBK_WV(T, PV, NTW)                                                                        \
    {                                                                                             \
        auto kern = projbwd_wave_kernel<T, PV, NTW>;                                              \
        if (wv_lds > 65536) {                                                                     \
            hipError_t e = hipFuncSetAttribute((const void *)kern,                                \
                                               hipFuncAttributeMaxDynamicSharedMemorySize,        \
                                               (int)wv_lds);                                      \
            if (e != hipSuccess)                                                                  \
                return e;                                                                         \
        }                                                                                         \
        hipLaunchKernelGGL(kern, grid, dim3(256), wv_lds, st, a);                                 \
        return hipGetLastError();                                                                 \
    }
#define MBK_WV_N(T, PV)                                                                           \
    {                                                                                             \
        if (ntw == 1)                                                                             \
            MBK_WV(T, PV, 1)                                                                      \
        if (ntw == 2)                                                                             \
            MBK_WV(T, PV, 2)                                                                      \
        MBK_WV(T, PV, 3)                                                                          \
    }
        if (bf16) {
            if (sc.pro == PRO_NONE)
                MBK_WV_N(bf16_t, PRO_NONE)
            MBK_WV_N(bf16_t, PRO_BNSWISH_GATE)
        }
        if (sc.pro == PRO_NONE)
            MBK_WV_N(float, PRO_NONE)
        MBK_WV_N(float, PRO_BNSWISH_GATE)
#undef MBK_WV_N
#undef MBK_WV
    }
#define MBK_CASE(T, PV)                                                                           \
    {                                                                                             \
        auto kern = wgrad_lt_kernel<T, 1, PRO_BNBWD, PV, true>;                                   \
        hipError_t e = hipFuncSetAttribute((const void *)kern,                                    \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess)                                                                      \
            return e;                                                                             \
        hipLaunchKernelGGL(kern, grid, block, lds, st, a);                                        \
        return hipGetLastError();                                                                 \
    }
    if (bf16) {
        if (sc.pro == PRO_NONE)
            MBK_CASE(bf16_t, PRO_NONE)
        MBK_CASE(bf16_t, PRO_BNSWISH_GATE)
    }
    if (sc.pro == PRO_NONE)
        MBK_CASE(float, PRO_NONE)
    MBK_CASE(float, PRO_BNSWISH_GATE)
#undef MBK_CASE
}

// kernels_x3.hip
bool bwd1x1_x3_supported(int Cw, int Cn, int HW);
hipError_t launch_bwd1x1_x3(int N, int Cw, int Cn, int HW, const Operand &de, const void *xin,
                            const void *w, void *dx, const void *res, float *partial, int splits,
                            hipStream_t st);

#ifndef MBK_X3B
#define MBK_X3B 1
#endif
// which matrix-core form serves the fused backward of this shape: 1 = fp32 MFMA (bwd1x1_lt),
// 3 = three bf16 planes (bwd1x1_x3); 0: the shape is not fused
int bwd1x1_fused_engine(bool bf16, int N, int Cw, int Cn, int HW)
{
    int splits;
    if (!bwd1x1_fused_plan(N, Cw, Cn, HW, &splits))
        return 0;
    return (!bf16 && MBK_X3B && bwd1x1_x3_supported(Cw, Cn, HW)) ? 3 : 1; // (bf16 storage: fp32 MFMA)
}

bool bwd1x1_fused_plan(int N, int Cw, int Cn, int HW, int *splits)
{
    bool swap;
    // the narrow side must be the convolution's input and fit one 32-row tile (two tiles would
    // need more registers and LDS than two workgroups per CU leave); other shapes go the
    // ordinary way, as two kernels
    return Cn <= 32 && Cn < Cw && wgrad_cl_plan(Cw, Cn, N, HW, &swap, splits) && swap;
}

hipError_t launch_bwd1x1_fused(bool bf16, int N, int Cw, int Cn, int HW, const Operand &de,
                               const void *xin, const void *w, void *dx, const void *res,
                               float *partial, int *splits_out, hipStream_t st)
{
    int splits;
    if (!bwd1x1_fused_plan(N, Cw, Cn, HW, &splits) || de.pro != PRO_BNBWD)
        return hipErrorInvalidValue;
    // fp32, at most 16 -> 96 channels: the wave-per-chunk kernel on the bf16 matrix cores
    // (same partial-tile layout and count)
    if (bwd1x1_fused_engine(bf16, N, Cw, Cn, HW) == 3) {
        *splits_out = splits;
        return launch_bwd1x1_x3(N, Cw, Cn, HW, de, xin, w, dx, res, partial, splits, st);
    }
    Bwd1x1Args b = {};
    WgradClArgs &a = b.g;
    a.N = N;
    a.Ma = Cn;
    a.Mb = Cw;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    a.numChunks = (int)((a.Q + 31u) / 32u);
    a.chunksPerWg = (a.numChunks + splits - 1) / splits;
    a.divHW = make_div((uint32_t)HW);
    a.u0 = xin;
    a.v0 = de.p0;
    a.v1 = de.p1;
    a.vc0 = de.c0;
    a.vc1 = de.c1;
    a.vc2 = de.c2;
    a.sOa = 1; // the caller's dW is [Cw][Cn] row-major
    a.sOb = Cn;
    a.partial = partial;
    b.w = w;
    b.dx = dx;
    b.res = res;
    *splits_out = splits;
    const int mta = (Cn + 31) / 32, mtb = (Cw + 31) / 32;
    const int nw = mtb < 4 ? 4 : mtb; // >= 256 threads stage x and finish dx
    const size_t lds = sizeof(float) * (kLtPitch * 32 * (2 * mta + nw + (size_t)nw * mta) +
                                        (size_t)nw * mta * 16 * 64 + 3 * 32 * nw);
    // Deal the data gradient's ceil(Cw/2) contraction steps out to the wavefronts so that the
    // SIMDs (wavefront t runs on SIMD t % 4) end up with equal MFMA counts; a wavefront with a
    // weight-gradient tile already has 16 per narrow tile.
    {
        const int K = (Cw + 1) / 2;
        int load[4] = {0, 0, 0, 0}, cnt[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int t = 0; t < nw; ++t)
            if (t < mtb)
                load[t % 4] += 16;
        for (int k = 0; k < K; ++k) { // one step at a time to the least loaded SIMD's least loaded wave
            int sbest = 0;
            for (int sd = 1; sd < 4; ++sd)
                if (load[sd] < load[sbest])
                    sbest = sd;
            int tbest = sbest;
            for (int t = sbest; t < nw; t += 4)
                if (cnt[t] < cnt[tbest])
                    tbest = t;
            ++cnt[tbest];
            ++load[sbest];
        }
        b.kbeg[0] = 0;
        for (int t = 0; t < 8; ++t)
            b.kbeg[t + 1] = b.kbeg[t] + (t < nw ? cnt[t] : 0);
    }
    dim3 grid((unsigned)splits), block((unsigned)(64 * nw));
#define MBK_CASE(T, MTA)                                                                          \
    {                                                                                             \
        hipError_t e = hipFuncSetAttribute((const void *)bwd1x1_lt_kernel<T, MTA>,                \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess)                                                                      \
            return e;                                                                             \
        hipLaunchKernelGGL((bwd1x1_lt_kernel<T, MTA>), grid, block, lds, st, b);                  \
        return hipGetLastError();                                                                 \
    }
    if (bf16)
        MBK_CASE(bf16_t, 1)
    MBK_CASE(float, 1)
#undef MBK_CASE
}

} // namespace mbk
