// fp32 1x1 convolutions and weight gradients of the wide blocks on the bf16 matrix cores.
//
// An fp32 MFMA (v_mfma_f32_32x32x2_f32) runs at the rate of the vector ALU and blocks it; the
// bf16 MFMA (v_mfma_f32_32x32x16_bf16) does sixteen times the work per cycle and runs beside
// the vector ALU.  An fp32 value is the exact sum of three bf16 values (8 + 8 + 8 significant
// bits: h = bf16(x), m = bf16(x - h), l = bf16(x - h - m), every subtraction exact), and a
// product of two bf16 values is exact in fp32, so
//     a*b = ah*bh + (ah*bm + am*bh) + (am*bm + ah*bl + al*bh) + O(2^-24 |a*b|):
// six bf16 MFMAs with fp32 accumulation reproduce the fp32 contraction to fp32 rounding level
// (the dropped terms are of the size of one fp32 rounding of the product) at 6/16 of the fp32
// MFMA's matrix-core time, and that time overlaps with the staging arithmetic.  Storage stays
// fp32 in HBM; the three planes of an activation exist in LDS only, those of the conv weights
// are written once per forward pass (x3_prep_kernel) in the order the kernels keep them in LDS.
//
// Same decomposition as kernels_big.hip / kernels_bf.hip: flattened batch (column q = n*HW +
// pixel), 64 x 64 output tiles per workgroup of four wavefronts, the contraction 32 at a time
// through two LDS buffers fed from a two-slot register ring, fixed-order split reductions.
// Operand layout of the instruction: lane l holds, of A, row l%32 and the contraction indices
// 8*(l/32)..+7; of B, column l%32 and the same indices; so both LDS tiles are [row or column][k]
// with k contiguous (pitch BK+8 halfwords = 80 bytes: 16-byte reads of a quarter wavefront fall
// on distinct banks), one such tile per plane.
#include <algorithm>
#include "mbconv_dev.h"
#include "mbconv_launch.h"


namespace mbk {

typedef float float16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct X3Operand {
    const float *p0, *p1;
    const float *c0, *c1, *c2, *gate;
};

// (x0, x1) -> three words, each the bf16 pair (plane value of x0 in bits 0-15, of x1 in 16-31)
__device__ __forceinline__ void x3_split2(float x0, float x1, uint32_t (&w)[3])
{
    w[0] = bf16_pack2(x0, x1);
    float r0 = x0 - __uint_as_float(w[0] << 16), r1 = x1 - __uint_as_float(w[0] & 0xffff0000u);
    w[1] = bf16_pack2(r0, r1);
    r0 -= __uint_as_float(w[1] << 16);
    r1 -= __uint_as_float(w[1] & 0xffff0000u);
    w[2] = bf16_pack2(r0, r1);
}

template <int PRO>
__device__ __forceinline__ float x3_apply(float v0, float v1, float k0, float k1, float k2)
{
    if (PRO == PRO_NONE)
        return v0;
    if (PRO == PRO_BNSWISH_GATE)
        return actf(fmaf(v0, k0, k1)) * k2;
    return fmaf(k0, v0, fmaf(k1, v1, k2));
}

__device__ __forceinline__ void x3_ld4(const float *p, size_t i, float (&v)[4])
{
    const float4 t = *reinterpret_cast<const float4 *>(p + i);
    v[0] = t.x;
    v[1] = t.y;
    v[2] = t.z;
    v[3] = t.w;
}
// four consecutive floats at an address that is only 4-byte aligned (pixel runs of planes whose
// size is not a multiple of four)
typedef float float4u __attribute__((ext_vector_type(4), aligned(4)));
__device__ __forceinline__ void x3_ld4u(const float *p, size_t i, float (&v)[4])
{
    const float4u t = *reinterpret_cast<const float4u *>(p + i);
    v[0] = t[0];
    v[1] = t[1];
    v[2] = t[2];
    v[3] = t[3];
}

// Halfword offset of element (row, k) in a [rows][BK = 32] plane of pitch 40 halfwords (80 bytes).
// The four 16-byte groups of a row are permuted by bits 4-5 of the row: the transposing stores
// (a wavefront writes one 32-bit k pair to each of 16 rows that are four apart, or to 64
// consecutive rows) then fall on 64 distinct banks instead of 16, and the 16-byte reads of 16
// consecutive rows stay conflict-free.
__device__ __forceinline__ int x3_at(int row, int k)
{
    return row * 40 + ((((k >> 3) ^ (row >> 4)) & 3) << 3) + (k & 7);
}

__device__ __forceinline__ bf16x8 x3_lds8(const uint16_t *p)
{
    return *reinterpret_cast<const bf16x8 *>(p);
}

// acc += a*b for the three-plane operands (small terms first)
__device__ __forceinline__ float16v x3_mfma6(const bf16x8 (&a)[3], const bf16x8 (&b)[3], float16v acc)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2], b[0], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[2], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[1], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[0], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[1], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], acc, 0, 0, 0);
    return acc;
}

// ---- weight images -------------------------------------------------------------------------
// The A operand of a convolution (rows m, contraction index k) as bf16 planes, cut into tiles
// of 64 rows x 32 k: tile (mt, ch), plane pl starts at halfword ((mt*CH + ch)*3 + pl)*2048 and
// holds element (row, k) at x3_img_at(row, k): rows of 64 bytes whose four 16-byte groups are
// permuted by bits 2-3 of the row, which keeps the 16-byte fragment reads of 16 consecutive
// rows on distinct banks without padding.  A workgroup copies a tile to LDS as it is (one 16-byte
// piece per thread and plane).  Rows and k past the end are zeros.
__device__ __forceinline__ int x3_img_at(int row, int k)
{
    return row * 32 + ((((k >> 3) ^ (row >> 2)) & 3) << 3) + (k & 7);
}

struct X3PrepSet {
    const float *w; // A(m, k) = w[m*sm + k*sk]
    int M, K, sm, sk;
    uint16_t *img;
    int CH, firstTile;
    int lane_order; // the tile's arrangement: 0 as described above (conv_x3), 1 for conv_xw
};
struct X3PrepArgs {
    X3PrepSet s[4];
    int nsets;
};

// one workgroup per tile: thread -> (row tid/4, eight k at 8*(tid%4))
__global__ __launch_bounds__(256) void x3_prep_kernel(X3PrepArgs a)
{
    int si = 0;
#pragma unroll
    for (int i = 1; i < 4; ++i)
        if (i < a.nsets && (int)blockIdx.x >= a.s[i].firstTile)
            si = i;
    const X3PrepSet S = a.s[si];
    const int local = blockIdx.x - S.firstTile, mt = local / S.CH, ch = local % S.CH;
    const int tid = threadIdx.x, r = tid >> 2, g = tid & 3;
    const int m = mt * 64 + r, k0 = ch * 32 + 8 * g;
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int k = k0 + j;
        v[j] = (m < S.M && k < S.K) ? S.w[(size_t)m * S.sm + (size_t)k * S.sk] : 0.f;
    }
    uint32_t w[4][3];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        x3_split2(v[2 * j], v[2 * j + 1], w[j]);
    uint16_t *tile = S.img + ((size_t)mt * S.CH + ch) * 3 * 2048;
    // lane order: the tile as four 16-row MFMA operands, [row tile][plane][lane] with lane =
    // row % 16 + 16 * (k / 8): a wavefront reads an operand as 64 consecutive 16-byte pieces
    const int at1 = (((r >> 4) * 3) * 64 + (r & 15) + 16 * g) * 8;
#pragma unroll
    for (int pl = 0; pl < 3; ++pl)
        *reinterpret_cast<uint4 *>(tile + (S.lane_order ? at1 + pl * 512 : pl * 2048 + x3_img_at(r, 8 * g))) =
            make_uint4(w[0][pl], w[1][pl], w[2][pl], w[3][pl]);
}

size_t x3_weight_image_bytes(int M, int K)
{
    return (size_t)((M + 63) / 64) * ((K + 31) / 32) * 3 * 2048 * sizeof(uint16_t);
}

// Writes up to four images in one launch; set i: A(m,k) = w[i][m*sm[i] + k*sk[i]], M[i] x K[i].
hipError_t launch_x3_prep(int nsets, const float *const *w, const int *M, const int *K, const int *sm,
                          const int *sk, void *const *img, const int *lane_order, hipStream_t st)
{
    if (nsets < 1 || nsets > 4)
        return hipErrorInvalidValue;
    X3PrepArgs a = {};
    int tiles = 0;
    for (int i = 0; i < nsets; ++i) {
        a.s[i].w = w[i];
        a.s[i].M = M[i];
        a.s[i].K = K[i];
        a.s[i].sm = sm[i];
        a.s[i].sk = sk[i];
        a.s[i].img = (uint16_t *)img[i];
        a.s[i].lane_order = lane_order[i];
        a.s[i].CH = (K[i] + 31) / 32;
        a.s[i].firstTile = tiles;
        tiles += ((M[i] + 63) / 64) * a.s[i].CH;
    }
    a.nsets = nsets;
    hipLaunchKernelGGL(x3_prep_kernel, dim3((unsigned)tiles), dim3(256), 0, st, a);
    return hipGetLastError();
}

// ---- convolution ---------------------------------------------------------------------------
struct X3ConvArgs {
    int M, K, HW;
    uint32_t Q;
    FastDiv divHW;
    const uint16_t *img; // weight image of this convolution's A operand
    int CH;              // its chunks of 32 along k
    X3Operand B;
    float *out;
    const float *res;
    float *psum, *psq;
    int QT, MT;
    float *partial;
    int chunksPerSplit;
};

// out[n,m,pix] = sum_k A(m,k) * op(B)[n,k,pix], A given as a weight image.  Requirements
// (checked by the host): K % 8 == 0, M % 4 == 0, HW % 4 == 0.
//
// PT (plane tiles, for planes of at most 64 pixels whose size is not a multiple of four: the
// 7x7 stages): a tile's 64 columns are the pixels of ONE image (QT = N), columns past the plane
// are zeros.  Pixel runs then never straddle an image; the last, partial run of a plane is read
// and written four pixels wide starting at HW-4, overlapping the run before it with identical
// values, so every access stays 16 bytes wide (4-byte aligned) and inside its plane.
//
// Persistent workgroups.  Output tiles are dealt out per XCD (blockIdx.x mod 8): XCD x owns the
// pixel tiles qt = x, x+8, ... with all their row tiles, so the workgroups that read the same
// activation tile share an L2; workgroup i of the XCD's Gx takes that list's tiles i, i+Gx, ...
// The (tile, chunk) items of a workgroup form one stream: the register ring prefetches two
// items ahead across tile boundaries, so the first chunks of the next tile are in flight while
// the current tile's results leave, and the start-up latency is paid once per workgroup.
template <int PRO, int EPI, bool PT>
__global__ __launch_bounds__(256) void conv_x3_kernel(X3ConvArgs a)
{
    constexpr int BM = 64, BP = 64, BK = 32, PK = BK + 8, PC = BP + 4;
    static_assert(PK == 40, "x3_at assumes a pitch of 40 halfwords");
    constexpr int kPlaneA = BM * BK, kPlaneB = BP * PK; // halfwords
    constexpr int kBuf = 3 * (kPlaneA + kPlaneB);
    // one operand buffer during the contraction, the fp32 output tile after it
    __shared__ __attribute__((aligned(16))) uint16_t smem[kBuf];
    static_assert(kBuf * 2 >= 64 * PC * 4, "output tile must fit into the operand buffer");
    float(*Ct)[PC] = reinterpret_cast<float(*)[PC]>(smem);
    auto As = [&](int pl) __attribute__((always_inline)) { return smem + pl * kPlaneA; };
    auto Bs = [&](int pl) __attribute__((always_inline)) { return smem + 3 * kPlaneA + pl * kPlaneB; };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wp = wave & 1;
    const int xcd = blockIdx.x & 7, wi = blockIdx.x >> 3, Gx = gridDim.x >> 3;
    const int nTx = a.QT > xcd ? ((a.QT - xcd + 7) >> 3) * a.MT : 0; // tiles of this XCD
    if (wi >= nTx)
        return;
    const int nT = (nTx - wi + Gx - 1) / Gx; // tiles of this workgroup
    int cbeg = 0, cend = (a.K + BK - 1) / BK;
    if (EPI == EPI_PARTIAL) {
        cbeg = blockIdx.y * a.chunksPerSplit;
        cend = min(cbeg + a.chunksPerSplit, cend);
    }
    const int nch = cend - cbeg, total = nT * nch;
    if (nch <= 0) // cannot happen with the host's split plan; keeps every image access in bounds
        return;

    // ---- prefetch cursor: the item the next load takes, and what depends on its tile ----
    // this thread's pixel run (tile columns brow .. brow+3) and k pair of a B chunk
    const int c0 = 4 * (tid & 15), kp = tid >> 4;
    const bool runIn = !PT || c0 < a.HW;                            // the run holds pixels of the plane
    const int brow = (PT && runIn && c0 + 4 > a.HW) ? a.HW - 4 : c0; // the partial run starts at HW-4
    int pk = 0, pc = cbeg, pmt = 0;
    bool bvalid = false;
    uint32_t bn = 0;
    size_t bbase = 0;
    auto set_ptile = [&](int k) __attribute__((always_inline)) {
        const int t = wi + min(k, nT - 1) * Gx; // past the last tile: the last one again (never consumed)
        const int qt = xcd + 8 * (t / a.MT);
        pmt = t - (t / a.MT) * a.MT;
        if (PT) {
            bvalid = runIn;
            bn = (uint32_t)qt;
            bbase = (size_t)bn * a.K * a.HW + (runIn ? brow : 0);
        } else {
            const uint32_t qb = (uint32_t)qt * BP + (uint32_t)c0;
            bvalid = qb < a.Q;
            bn = bvalid ? fdiv(qb, a.divHW) : 0u;
            bbase = (size_t)bn * a.K * a.HW + (bvalid ? qb - bn * (uint32_t)a.HW : 0u);
        }
    };
    auto advance = [&]() __attribute__((always_inline)) {
        if (++pc == cend) { // uniform over the workgroup; no memory access inside
            pc = cbeg;
            set_ptile(++pk);
        }
    };

    // Staged items live in a ring of two register slots: item j is loaded during iteration j-2
    // and written to LDS at the end of iteration j-1.  All loads are unconditional (indices
    // clamped into the tensor) and validity is an AND mask applied on the way into LDS, so no
    // branch and no use of loaded data sits between a load and the MFMAs it should overlap.
    //
    // A: the tile's three planes are copied as they are, 16 bytes per thread and plane.
    u32x4 ra[2][3];
    // B: thread -> (four pixels at 4*(tid%16), k pair tid/16); the pair of a pixel is one 32-bit
    // LDS store per plane.
    float rb0[2][2][4], rb1[2][2][PRO == PRO_BNBWD ? 4 : 1];
    float bk0[2][2], bk1[2][2], bk2[2][2];
    uint32_t rbok[2][2];
    auto load = [&](int s) __attribute__((always_inline)) {
        const uint16_t *tile = a.img + ((size_t)pmt * a.CH + pc) * 3 * kPlaneA;
#pragma unroll
        for (int pl = 0; pl < 3; ++pl)
            ra[s][pl] = *reinterpret_cast<const u32x4 *>(tile + pl * kPlaneA + 8 * tid);
        const int k0 = pc * BK;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int k = k0 + 2 * kp + j, kc = min(k, a.K - 1);
            rbok[s][j] = (bvalid && k < a.K) ? 0xffffffffu : 0u;
            if (PT)
                x3_ld4u(a.B.p0, bbase + (size_t)kc * a.HW, rb0[s][j]);
            else
                x3_ld4(a.B.p0, bbase + (size_t)kc * a.HW, rb0[s][j]);
            if constexpr (PRO == PRO_BNBWD) {
                if (PT)
                    x3_ld4u(a.B.p1, bbase + (size_t)kc * a.HW, rb1[s][j]);
                else
                    x3_ld4(a.B.p1, bbase + (size_t)kc * a.HW, rb1[s][j]);
            }
            if (PRO != PRO_NONE) {
                bk0[s][j] = a.B.c0[kc];
                bk1[s][j] = a.B.c1[kc];
                bk2[s][j] = PRO == PRO_BNBWD ? a.B.c2[kc] : a.B.gate[(size_t)bn * a.K + kc];
            }
        }
    };
    auto store = [&](int s) __attribute__((always_inline)) {
#pragma unroll
        for (int pl = 0; pl < 3; ++pl)
            *reinterpret_cast<u32x4 *>(As(pl) + 8 * tid) = ra[s][pl];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float v[2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
                v[j] = and_mask(x3_apply<PRO>(rb0[s][j][r], rb1[s][j][PRO == PRO_BNBWD ? r : 0], bk0[s][j],
                                              bk1[s][j], bk2[s][j]),
                                rbok[s][j]);
            uint32_t w[3];
            x3_split2(v[0], v[1], w);
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
                *reinterpret_cast<uint32_t *>(Bs(pl) + x3_at(brow + r, 2 * kp)) = w[pl];
        }
    };

    float16v acc;
#pragma unroll
    for (int r = 0; r < 16; ++r)
        acc[r] = 0.f;

    // ---- results of the current tile; register r of lane l is row 8*(r/4)+4*(l/32)+r%4, column l%32 ----
    auto epilogue = [&](int ck) __attribute__((always_inline)) {
        const int t = wi + ck * Gx;
        const int qt = xcd + 8 * (t / a.MT), m0 = (t - (t / a.MT) * a.MT) * BM;
        const uint32_t q0 = PT ? (uint32_t)qt * (uint32_t)a.HW : (uint32_t)qt * BP; // first pixel of the tile
        if constexpr (EPI != EPI_PARTIAL) {
            // Through LDS, so that 16 lanes own the pixels of one output row: 16-byte accesses, one
            // pixel-index division per thread, and a row's BN statistics summed inside those 16
            // lanes.  (The chunk's barrier has passed: the operand buffer is free.)
            const int pg = tid & 15;
            bool valid;
            uint32_t n, pix;
            int fresh = 0; // first element of the run that no other run covers
            if (PT) {
                valid = runIn;
                n = (uint32_t)qt;
                pix = runIn ? (uint32_t)brow : 0u;
                fresh = runIn ? c0 - brow : 0;
            } else {
                const uint32_t q = q0 + 4u * pg;
                valid = q < a.Q;
                n = valid ? fdiv(q, a.divHW) : 0u;
                pix = valid ? q - n * (uint32_t)a.HW : 0u;
            }
#pragma unroll
            for (int r = 0; r < 16; ++r)
                Ct[wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)][wp * 32 + (lane & 31)] = acc[r];
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = (tid >> 4) + 16 * i, m = m0 + row;
                const bool ok = valid && m < a.M;
                float v[4];
                if (PT) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        v[j] = Ct[row][(runIn ? brow : 0) + j];
                } else {
                    const float4 c = *reinterpret_cast<const float4 *>(&Ct[row][4 * pg]);
                    v[0] = c.x;
                    v[1] = c.y;
                    v[2] = c.z;
                    v[3] = c.w;
                }
                const size_t idx = ((size_t)n * a.M + min(m, a.M - 1)) * a.HW + pix;
                float rr[4] = {0.f, 0.f, 0.f, 0.f};
                if (EPI == EPI_RES || (EPI == EPI_AFFINE && a.res)) {
                    if (PT)
                        x3_ld4u(a.res, idx, rr);
                    else
                        x3_ld4(a.res, idx, rr);
                }
                if (EPI == EPI_RES) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        v[j] += rr[j];
                }
                if (EPI == EPI_AFFINE) { // psum / psq carry the row's scale and shift
                    const float osc = a.psum[min(m, a.M - 1)], osh = a.psq[min(m, a.M - 1)];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        v[j] = fmaf(v[j], osc, osh) + rr[j];
                }
                if (ok) {
                    if (PT) {
                        float4u o;
                        o[0] = v[0];
                        o[1] = v[1];
                        o[2] = v[2];
                        o[3] = v[3];
                        *reinterpret_cast<float4u *>(a.out + idx) = o;
                    } else {
                        *reinterpret_cast<float4 *>(a.out + idx) = make_float4(v[0], v[1], v[2], v[3]);
                    }
                }
                if (EPI == EPI_STATS) {
                    float s1 = 0.f, s2 = 0.f;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float sv = (ok && j >= fresh) ? v[j] : 0.f;
                        s1 += sv;
                        s2 = fmaf(sv, sv, s2);
                    }
                    s1 = row16_sum(s1);
                    s2 = row16_sum(s2);
                    if (pg == 0 && m < a.M) {
                        a.psum[(size_t)m * a.QT + qt] = s1;
                        a.psq[(size_t)m * a.QT + qt] = s2;
                    }
                }
            }
        } else {
            // a split contraction: the raw partial tile, lanes along the pixels
            const int col = wp * 32 + (lane & 31);
            const uint32_t q = q0 + (uint32_t)col;
            const bool valid = PT ? col < a.HW : q < a.Q;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (valid && m < a.M)
                    a.partial[((size_t)blockIdx.y * a.M + m) * a.Q + q] = acc[r];
            }
        }
    };

    // PT: tile columns past the plane must read as zeros, and the pixel runs do not cover all of
    // them (the partial run starts early); they are cleared before the first item and again after
    // every output tile, which passes through the same LDS.  (A store and a barrier follow.)
    auto zero_pad = [&]() __attribute__((always_inline)) {
        if (PT) {
            for (int i = tid; i < 3 * BP * 4; i += 256) {
                const int pl = i / (BP * 4), row = (i >> 2) & (BP - 1), g = i & 3;
                if (row >= a.HW)
                    *reinterpret_cast<uint4 *>(Bs(pl) + row * PK + 8 * g) = make_uint4(0u, 0u, 0u, 0u);
            }
        }
    };
    zero_pad();
    set_ptile(0);
    load(0);
    advance();
    load(1);
    advance();
    store(0);
    __syncthreads();
    int ck = 0, cj = 0; // current tile of this workgroup, chunk within it
    auto body = [&](int u) __attribute__((always_inline)) {
        load(u); // slot u is free: its item went to LDS last iteration
        advance();
        __builtin_amdgcn_sched_barrier(0); // loads first, then the MFMAs, then the staging arithmetic
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            bf16x8 av[3], bv[3];
            const int ko = 16 * s + 8 * (lane >> 5);
#pragma unroll
            for (int pl = 0; pl < 3; ++pl) {
                av[pl] = x3_lds8(As(pl) + x3_img_at(wm * 32 + (lane & 31), ko));
                bv[pl] = x3_lds8(Bs(pl) + x3_at(wp * 32 + (lane & 31), ko));
            }
            acc = x3_mfma6(av, bv, acc);
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads(); // every wavefront has read the chunk
        if (++cj == nch) { // uniform: the tile is complete
            epilogue(ck);
            __syncthreads(); // the output tile has left LDS
            zero_pad();
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[r] = 0.f;
            cj = 0;
            ++ck;
        }
        store(u ^ 1); // past the last item: a repeated item that is never consumed
        __syncthreads();
    };
    int it = 0;
    for (; it + 1 < total; it += 2) {
        body(0);
        body(1);
    }
    if (it < total)
        body(0);
}

// Plan: 64 x 64 tiles; the contraction is split when the tiles alone cannot fill the chip
// (`qtiles` is then the second stage's count of statistics partials per row).
bool x3_conv_plan(int N, int M, int K, int HW, int *qtiles, int *splits)
{
    const long long Q = (long long)N * HW;
    if (K % 8 != 0 || M % 4 != 0 || Q >= (1ll << 31) || K < 32 || M < 32)
        return false;
    // planes whose size is not a multiple of four: one image per tile if a plane fits (the 7x7
    // stages); larger ones stay with kernels_big.hip
    const bool pt = HW % 4 != 0;
    if (pt && (HW > 64 || HW < 4))
        return false;
    *qtiles = pt ? N : (int)((Q + 63) / 64);
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

size_t x3_conv_splitk_floats(int N, int M, int K, int HW)
{
    int qtiles, splits;
    if (!x3_conv_plan(N, M, K, HW, &qtiles, &splits) || splits == 1)
        return 0;
    return (size_t)splits * M * N * HW;
}

// kernels_big.hip
hipError_t launch_splitk_finish_f32(const float *partial, int S, int M, uint32_t Q, int HW, void *out,
                                    const void *res, int epi, float *psum, float *psq, int NT,
                                    hipStream_t st);

hipError_t launch_x3_conv1x1(int N, int M, int K, int HW, const void *wimg, const Operand &B,
                             void *out, int epi, const void *res, float *psum, float *psq,
                             float *splitk_ws, hipStream_t st)
{
    int qtiles, splits;
    if (!x3_conv_plan(N, M, K, HW, &qtiles, &splits) || !wimg)
        return hipErrorInvalidValue;
    if (splits > 1 && (!splitk_ws || epi == EPI_AFFINE))
        return hipErrorInvalidValue;
    X3ConvArgs a;
    a.M = M;
    a.K = K;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    a.divHW = make_div((uint32_t)HW);
    a.img = (const uint16_t *)wimg;
    a.CH = (K + 31) / 32;
    a.B.p0 = (const float *)B.p0;
    a.B.p1 = (const float *)B.p1;
    a.B.c0 = B.c0;
    a.B.c1 = B.c1;
    a.B.c2 = B.c2;
    a.B.gate = B.gate;
    a.out = (float *)out;
    a.res = (const float *)res;
    a.psum = psum;
    a.psq = psq;
    const bool pt = HW % 4 != 0; // one image per tile
    a.QT = pt ? N : (int)((a.Q + 63u) / 64u);
    a.MT = (M + 63) / 64;
    a.partial = splitk_ws;
    const int chunks = (K + 31) / 32;
    a.chunksPerSplit = (chunks + splits - 1) / splits;
    // workgroups per XCD: every workgroup gets the same number of tiles (or one fewer), at most
    // about four workgroups per compute unit in all
    const int tilesPerXcd = ((a.QT + 7) / 8) * a.MT;
    const int cap = std::max(1, 128 / splits);
    const int rounds = (tilesPerXcd + cap - 1) / cap;
    const int gx = (tilesPerXcd + rounds - 1) / rounds;
    dim3 grid((unsigned)(8 * gx), (unsigned)splits);
    const int kepi = splits > 1 ? EPI_PARTIAL : epi;
    hipError_t e = hipErrorInvalidValue;
#define MBK_CASE(P, E)                                                                            \
    if (B.pro == P && kepi == E) {                                                                \
        if (pt)                                                                                   \
            hipLaunchKernelGGL((conv_x3_kernel<P, E, true>), grid, dim3(256), 0, st, a);          \
        else                                                                                      \
            hipLaunchKernelGGL((conv_x3_kernel<P, E, false>), grid, dim3(256), 0, st, a);         \
        e = hipGetLastError();                                                                    \
    }
    MBK_CASE(PRO_NONE, EPI_STATS)
    MBK_CASE(PRO_BNSWISH_GATE, EPI_STATS)
    MBK_CASE(PRO_BNBWD, EPI_NONE)
    MBK_CASE(PRO_BNBWD, EPI_RES)
    MBK_CASE(PRO_BNSWISH_GATE, EPI_AFFINE)
    MBK_CASE(PRO_NONE, EPI_PARTIAL)
    MBK_CASE(PRO_BNSWISH_GATE, EPI_PARTIAL)
    MBK_CASE(PRO_BNBWD, EPI_PARTIAL)
#undef MBK_CASE
    if (e != hipSuccess || splits == 1)
        return e;
    return launch_splitk_finish_f32(splitk_ws, splits, M, a.Q, HW, out, res, epi, psum, psq, qtiles, st);
}

// ---- weight gradient -------------------------------------------------------------------------
// dW[a,b] = sum_q op(U)[a,q] * op(V)[b,q].  Both operands are pixel-contiguous in memory, which
// is the [row][k] layout the instruction wants, so a run of four pixels goes through its
// prologue, is split and lands in LDS as one 8-byte store per plane.  A workgroup of eight
// wavefronts owns 128 rows of U by 128 rows of V (each wavefront 64 x 32) and a range of
// 32-pixel chunks; with the narrow operand inside one tile the wide one is staged, and sent
// through its prologue, once in the whole grid.  Chunks are loaded two iterations ahead into a
// ring of two register slots, so HBM stays busy while a chunk is split and multiplied.  The
// splits' partial tiles are added by a fixed-order second stage.
struct X3WgradArgs {
    int Ma, Mb, HW;
    uint32_t Q;
    int chunksPerSplit; // chunks of 32 pixels
    int tilesA, tilesB, splits;
    FastDiv divHW;
    X3Operand U, V;
    float *partial;
};

// what a thread keeps per operand for the whole kernel: rows rr + 64*i (i < NP) of the tile
template <int PRO, int NP>
struct X3RowConst {
    float k0[NP], k1[NP], k2[NP];
    uint32_t rmask[NP];
    __device__ __forceinline__ void init(const X3Operand &o, int row0, int rr, int M)
    {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int r = row0 + rr + 64 * i;
            rmask[i] = r < M ? 0xffffffffu : 0u;
            k0[i] = k1[i] = k2[i] = 0.f;
            if (PRO != PRO_NONE && r < M) {
                k0[i] = o.c0[r];
                k1[i] = o.c1[r];
                if (PRO == PRO_BNBWD)
                    k2[i] = o.c2[r];
            }
        }
    }
};
// one ring slot of an operand: the raw pixel runs (four pixels at 4*qg) of the thread's rows
template <int PRO, int NP>
struct X3RowData {
    float v0[NP][4], v1[NP][PRO == PRO_BNBWD ? 4 : 1];
    float g[NP];
    // n, pix: image and first pixel of the run (it lies inside one plane: HW % 4 == 0).  Both rows
    // load, also past the last row (clamped, masked on the way into LDS): a branch around a load
    // would make the loads behind it wait.
    __device__ __forceinline__ void load(const X3Operand &o, int row0, int rr, int M, int HW, uint32_t n,
                                         uint32_t pix)
    {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int r = min(row0 + rr + 64 * i, M - 1);
            const size_t idx = ((size_t)n * M + r) * HW + pix;
            x3_ld4(o.p0, idx, v0[i]);
            if constexpr (PRO == PRO_BNBWD)
                x3_ld4(o.p1, idx, v1[i]);
            if constexpr (PRO == PRO_BNSWISH_GATE)
                g[i] = o.gate[(size_t)n * M + r];
        }
    }
    // prologue, split, three 8-byte LDS stores per row
    __device__ __forceinline__ void store(const X3RowConst<PRO, NP> &c, uint16_t *planes, int rr, int qg,
                                          uint32_t qmask) const
    {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            float y[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                y[j] = and_mask(x3_apply<PRO>(v0[i][j], v1[i][PRO == PRO_BNBWD ? j : 0], c.k0[i], c.k1[i],
                                              PRO == PRO_BNSWISH_GATE ? g[i] : c.k2[i]),
                                qmask & c.rmask[i]);
            uint32_t w0[3], w1[3];
            x3_split2(y[0], y[1], w0);
            x3_split2(y[2], y[3], w1);
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
                *reinterpret_cast<uint2 *>(planes + pl * (NP * 64 * 32) + x3_img_at(rr + 64 * i, 4 * qg)) =
                    make_uint2(w0[pl], w1[pl]);
        }
    }
};

// VB: rows of the V tile, 128 or 64 (a narrow second operand: each wavefront then owns 32 x 32).
// TR: the partial tile is written transposed (the host swaps the operands when the first one is
// the narrow one).
// (`bid`: the workgroup's index within this weight gradient's grid; Us, Vs: LDS for three planes
// of 128 and of VB rows)
template <int PROU, int PROV, int VB, bool TR>
__device__ __forceinline__ void wgrad_x3_body(const X3WgradArgs &a, int bid, uint16_t *Us, uint16_t *Vs)
{
    constexpr int BQ = 32, kPlane = 128 * 32, kPlaneV = VB * 32; // planes in the layout of x3_img_at
    constexpr int NA = VB == 128 ? 2 : 1;                        // 32-row blocks of U per wavefront
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // first row of this wavefront's part of the U tile and of the V tile
    const int ua = VB == 128 ? 64 * (wave >> 2) : 32 * (wave >> 1);
    const int vb = VB == 128 ? 32 * (wave & 3) : 32 * (wave & 1);
    // workgroups that read the same pixels (all tiles of one split) run on the same XCD
    // (blockIdx.x mod 8), so the operand that several tiles share comes out of that XCD's L2
    const int xcd = bid & 7, slot = bid >> 3;
    const int tiles = a.tilesA * a.tilesB;
    const int split = (slot / tiles) * 8 + xcd, tile = slot % tiles;
    if (split >= a.splits)
        return;
    const int a0 = (tile % a.tilesA) * 128, b0 = (tile / a.tilesA) * VB;
    const int numChunks = (int)((a.Q + BQ - 1) / BQ);
    const int cbeg = split * a.chunksPerSplit;
    const int cend = min(cbeg + a.chunksPerSplit, numChunks);
    const int qg = tid & 7, rr = tid >> 3;
    X3RowConst<PROU, 2> cu;
    X3RowConst<PROV, VB / 64> cv;
    cu.init(a.U, a0, rr, a.Ma);
    cv.init(a.V, b0, rr, a.Mb);
    X3RowData<PROU, 2> du[2];
    X3RowData<PROV, VB / 64> dv[2];
    uint32_t qmask[2] = {0u, 0u};
    // unconditional clamped loads, validity as an AND mask on the way into LDS
    auto load = [&](int s, int chunk) __attribute__((always_inline)) {
        const uint32_t q = (uint32_t)chunk * BQ + 4u * qg;
        qmask[s] = q < a.Q ? 0xffffffffu : 0u; // HW % 4 == 0: the run of four lies in one image
        const uint32_t qc = qmask[s] ? q : 0u;
        const uint32_t n = fdiv(qc, a.divHW), pix = qc - n * (uint32_t)a.HW;
        du[s].load(a.U, a0, rr, a.Ma, a.HW, n, pix);
        dv[s].load(a.V, b0, rr, a.Mb, a.HW, n, pix);
    };
    auto store = [&](int s) __attribute__((always_inline)) {
        du[s].store(cu, Us, rr, qg, qmask[s]);
        dv[s].store(cv, Vs, rr, qg, qmask[s]);
    };

    float16v acc[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            acc[i][r] = 0.f;
    if (cbeg < cend) { // uniform over the workgroup; an empty split writes zeros
        load(0, cbeg);
        load(1, min(cbeg + 1, cend - 1));
        store(0);
        __syncthreads();
        auto step = [&](int u, int cc) __attribute__((always_inline)) {
            load(u, min(cc + 2, cend - 1)); // slot u is free: its chunk went to LDS last iteration
            // the loads are all issued before the MFMAs start and nothing that uses their data
            // moves up among the MFMAs (the scheduler would otherwise wait for them there)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < BQ / 16; ++s) {
                const int ko = 16 * s + 8 * (lane >> 5);
                bf16x8 av[NA][3], bv[3];
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) {
#pragma unroll
                    for (int i = 0; i < NA; ++i)
                        av[i][pl] = x3_lds8(Us + pl * kPlane + x3_img_at(ua + 32 * i + (lane & 31), ko));
                    bv[pl] = x3_lds8(Vs + pl * kPlaneV + x3_img_at(vb + (lane & 31), ko));
                }
#pragma unroll
                for (int i = 0; i < NA; ++i)
                    acc[i] = x3_mfma6(av[i], bv, acc[i]); // rows past the end are zeros
            }
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads(); // every wavefront has read the chunk
            store(u ^ 1);    // the repeated last chunk is stored but never consumed
            __syncthreads();
        };
        int cc = cbeg;
        for (; cc + 1 < cend; cc += 2) {
            step(0, cc);
            step(1, cc + 1);
        }
        if (cc < cend) // uniform over the workgroup
            step(0, cc);
    }
    float *dst = a.partial + (size_t)split * a.Ma * a.Mb;
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int ai = a0 + ua + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            const int bi = b0 + vb + (lane & 31);
            if (ai < a.Ma && bi < a.Mb)
                dst[TR ? (size_t)bi * a.Ma + ai : (size_t)ai * a.Mb + bi] = acc[i][r];
        }
}

template <int PROU, int PROV, int VB, bool TR>
__global__ __launch_bounds__(512) void wgrad_x3_kernel(X3WgradArgs a)
{
    __shared__ __attribute__((aligned(16))) uint16_t Us[3 * 128 * 32];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[3 * VB * 32];
    wgrad_x3_body<PROU, PROV, VB, TR>(a, (int)blockIdx.x, Us, Vs);
}

// The six forms of the kernel above, by number (x3_wgrad_variant).
template <int VAR>
__device__ __forceinline__ void wgrad_x3_variant(const X3WgradArgs &a, int bid, uint16_t *Us, uint16_t *Vs)
{
    if (VAR == 0)
        wgrad_x3_body<PRO_BNBWD, PRO_NONE, 128, false>(a, bid, Us, Vs);
    else if (VAR == 1)
        wgrad_x3_body<PRO_BNBWD, PRO_BNSWISH_GATE, 128, false>(a, bid, Us, Vs);
    else if (VAR == 2)
        wgrad_x3_body<PRO_BNBWD, PRO_NONE, 64, false>(a, bid, Us, Vs);
    else if (VAR == 3)
        wgrad_x3_body<PRO_BNBWD, PRO_BNSWISH_GATE, 64, false>(a, bid, Us, Vs);
    else if (VAR == 4)
        wgrad_x3_body<PRO_NONE, PRO_BNBWD, 64, true>(a, bid, Us, Vs);
    else
        wgrad_x3_body<PRO_BNSWISH_GATE, PRO_BNBWD, 64, true>(a, bid, Us, Vs);
}

// Two weight gradients in one launch (a block's projection and expansion conv: independent of
// each other, each about one workgroup per compute unit and bound by the latency of its own
// load-stage-multiply chain): the first gridA workgroups work on `a`, the others on `b`, and
// with at most 128 registers two workgroups, one of each, share a compute unit.
template <int VARA, int VARB>
__global__ __launch_bounds__(512, 4) void wgrad_x3_pair_kernel(X3WgradArgs a, X3WgradArgs b, int gridA)
{
    __shared__ __attribute__((aligned(16))) uint16_t Us[3 * 128 * 32];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[3 * 128 * 32];
    if ((int)blockIdx.x < gridA) // uniform over the workgroup
        wgrad_x3_variant<VARA>(a, (int)blockIdx.x, Us, Vs);
    else
        wgrad_x3_variant<VARB>(b, (int)blockIdx.x - gridA, Us, Vs);
}

// Tile and splits.  The wider operand gets 128-row tiles; the other one 128-row tiles, or one
// 64-row tile when it has at most 64 rows (and more than 32).  Splits of the contraction: about one workgroup (eight
// wavefronts) per compute unit, at least two chunks each.
bool x3_wgrad_plan(int Ma, int Mb, int N, int HW, int *splits)
{
    const long long Q = (long long)N * HW;
    // (planes whose size is not a multiple of four stay with kernels_big.hip: one-image chunks with
    // a shifted partial run measured slower there, 41 -> 52 us on 1152 x 192 channels at 7x7)
    // (a side of at most 32 channels belongs to the fused backward kernels of kernels_wave.hip,
    // which size their partial tiles by the plan of that file)
    if (Q >= (1ll << 31) || HW % 4 != 0 || std::min(Ma, Mb) <= 32 || std::max(Ma, Mb) < 64)
        return false;
    const int wide = std::max(Ma, Mb), narrow = std::min(Ma, Mb), vb = narrow <= 64 ? 64 : 128;
    const long long tiles = (long long)((wide + 127) / 128) * ((narrow + vb - 1) / vb);
    const long long chunks = (Q + 31) / 32;
    long long s = (256 + tiles - 1) / tiles; // 512 workgroups measured slower (twice the partial tiles)
    const long long smax = (chunks + 1) / 2;
    if (s > smax)
        s = smax;
    if (s < 1)
        s = 1;
    const long long per = (chunks + s - 1) / s;
    *splits = (int)((chunks + per - 1) / per);
    return true;
}

static X3Operand to_x3(const Operand &o)
{
    X3Operand d;
    d.p0 = (const float *)o.p0;
    d.p1 = (const float *)o.p1;
    d.c0 = o.c0;
    d.c1 = o.c1;
    d.c2 = o.c2;
    d.gate = o.gate;
    return d;
}

// Arguments, grid and kernel form (0..5, see wgrad_x3_variant) of one weight gradient.
static bool x3_wgrad_setup(int N, int Ma, int Mb, int HW, const Operand &U, const Operand &V,
                           float *partial, X3WgradArgs *out, unsigned *grid, int *variant, int *splits_out)
{
    int splits;
    if (!x3_wgrad_plan(Ma, Mb, N, HW, &splits))
        return false;
    // a narrow first operand: the kernel computes the transposed product and writes it transposed
    const bool swap = Ma < 64 && Mb >= 64;
    const int vb = std::min(Ma, Mb) <= 64 ? 64 : 128;
    X3WgradArgs a;
    a.Ma = swap ? Mb : Ma;
    a.Mb = swap ? Ma : Mb;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    const int chunks = (int)((a.Q + 31u) / 32u);
    a.chunksPerSplit = (chunks + splits - 1) / splits;
    a.divHW = make_div((uint32_t)HW);
    a.U = to_x3(swap ? V : U);
    a.V = to_x3(swap ? U : V);
    a.partial = partial;
    *splits_out = splits;
    a.tilesA = (a.Ma + 127) / 128;
    a.tilesB = (a.Mb + vb - 1) / vb;
    a.splits = splits;
    *grid = (unsigned)(((splits + 7) / 8) * 8 * a.tilesA * a.tilesB);
    const int pu = swap ? V.pro : U.pro, pv = swap ? U.pro : V.pro;
    int var = -1;
    if (!swap && pu == PRO_BNBWD && pv == PRO_NONE)
        var = vb == 128 ? 0 : 2;
    else if (!swap && pu == PRO_BNBWD && pv == PRO_BNSWISH_GATE)
        var = vb == 128 ? 1 : 3;
    else if (swap && vb == 64 && pu == PRO_NONE && pv == PRO_BNBWD)
        var = 4;
    else if (swap && vb == 64 && pu == PRO_BNSWISH_GATE && pv == PRO_BNBWD)
        var = 5;
    if (var < 0)
        return false;
    *out = a;
    *variant = var;
    return true;
}

hipError_t launch_x3_wgrad(int N, int Ma, int Mb, int HW, const Operand &U, const Operand &V,
                           float *partial, int *splits_out, hipStream_t st)
{
    X3WgradArgs a;
    unsigned grid;
    int var;
    if (!x3_wgrad_setup(N, Ma, Mb, HW, U, V, partial, &a, &grid, &var, splits_out))
        return hipErrorInvalidValue;
#define MBK_CASE(VAR, PU, PV, VB_, TR_)                                                           \
    if (var == VAR) {                                                                             \
        hipLaunchKernelGGL((wgrad_x3_kernel<PU, PV, VB_, TR_>), dim3(grid), dim3(512), 0, st, a); \
        return hipGetLastError();                                                                 \
    }
    MBK_CASE(0, PRO_BNBWD, PRO_NONE, 128, false)
    MBK_CASE(1, PRO_BNBWD, PRO_BNSWISH_GATE, 128, false)
    MBK_CASE(2, PRO_BNBWD, PRO_NONE, 64, false)
    MBK_CASE(3, PRO_BNBWD, PRO_BNSWISH_GATE, 64, false)
    MBK_CASE(4, PRO_NONE, PRO_BNBWD, 64, true)
    MBK_CASE(5, PRO_BNSWISH_GATE, PRO_BNBWD, 64, true)
#undef MBK_CASE
    return hipErrorInvalidValue;
}

// The projection conv's weight gradient (A: dp x sc) and the expansion conv's (B: de x x) in one
// launch.  Returns hipErrorNotSupported, nothing launched, when one of them is not a shape of
// this file or their forms are not a pair the launch has.
hipError_t launch_x3_wgrad_pair(int N, int MaA, int MbA, int HWA, const Operand &UA, const Operand &VA,
                                float *partialA, int *splitsA, int MaB, int MbB, int HWB,
                                const Operand &UB, const Operand &VB, float *partialB, int *splitsB,
                                hipStream_t st)
{
    X3WgradArgs a, b;
    unsigned ga, gb;
    int va, vb;
    if (!x3_wgrad_setup(N, MaA, MbA, HWA, UA, VA, partialA, &a, &ga, &va, splitsA) ||
        !x3_wgrad_setup(N, MaB, MbB, HWB, UB, VB, partialB, &b, &gb, &vb, splitsB))
        return hipErrorNotSupported;
#define MBK_CASE(VA_, VB_)                                                                        \
    if (va == VA_ && vb == VB_) {                                                                 \
        hipLaunchKernelGGL((wgrad_x3_pair_kernel<VA_, VB_>), dim3(ga + gb), dim3(512), 0, st, a, b, \
                           (int)ga);                                                              \
        return hipGetLastError();                                                                 \
    }
    // projection side: dp (BN backward) with the gated activation, 128- or 64-row tile, or
    // swapped; expansion side: de (BN backward) with the block's input, likewise
    MBK_CASE(1, 0)
    MBK_CASE(1, 2)
    MBK_CASE(3, 2)
    MBK_CASE(3, 0)
    MBK_CASE(5, 2)
    MBK_CASE(5, 0)
    MBK_CASE(1, 4)
    MBK_CASE(3, 4)
    MBK_CASE(5, 4)
#undef MBK_CASE
    return hipErrorNotSupported;
}

// ---- both gradients of a narrow -> wide 1x1 convolution, a wavefront per pixel chunk ---------
// The expansion conv's backward when its input has at most 16 channels and its output at most
// 96: dx = W^T de (+ dout) and dW = de x^T from one pass over de = c0*dy1 + c1*e + c2 (BN1's
// backward applied on the way in), the two widest tensors of the block.  Same fusion as
// bwd1x1_lt in kernels_wave.hip (section "Guided Optimization Case Study: EfficientNet": the
// consumers of a tensor fused), rebuilt around what bounds that kernel, two workgroup barriers and
// a VALU-rate fp32 MFMA phase per 32-pixel chunk:
//   - a wavefront owns whole chunks of 32 pixels (chunk = 4*workgroup + wavefront, stride
//     4*grid); nothing crosses wavefronts inside the loop, so there is no barrier in it;
//   - lane (r = lane%16, g = lane/16) loads pixels 2r and 2r+1 of the chunk for the channels
//     32s + 8g .. +7 of every 32-channel step s, eight bytes at a time: sixteen consecutive lanes
//     read a whole 128-byte line (lanes that hold different ROWS of a tile, the layout the weight
//     gradient would take from registers, cost the address unit a cache line per lane: measured,
//     161 us on 16 -> 96 channels and 803 k pixels), and eight channels of one pixel are
//     exactly the B operand of v_mfma_f32_16x16x32_bf16 for the data gradient (column = pixel:
//     one tile for the even pixels, one for the odd; contraction = channels), whose A operand,
//     W^T, waits in registers: the data gradient needs no LDS;
//   - the weight gradient contracts over pixels, so each 32-channel step goes through LDS once,
//     transposed: [channel][pixel] bf16 planes, the lane's two pixels of a channel as one 32-bit
//     store, read back 16 bytes per lane as the A operand (row = channel); x takes the same route
//     once per chunk;
//   - the next chunk's values of a step are requested as soon as this chunk's have been
//     consumed, so they travel during the rest of the chunk's arithmetic.
// fp32 operands are split into three bf16 planes as everywhere in this file.  The four
// wavefronts' weight-gradient tiles are added in wavefront order at the end, the workgroups'
// partial tiles by reduce_splits: fixed order, no atomics.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

struct X3Bwd1x1Args {
    int Cn, Cw, HW;
    uint32_t Q;
    int numChunks;
    FastDiv divHW;
    const float *x, *dy, *e;   // [N][Cn][HW]; [N][Cw][HW] twice
    const float *c0, *c1, *c2; // [Cw]: de = c0*dy + c1*e + c2
    const float *w;            // [Cw][Cn]
    float *dx;                 // [N][Cn][HW]
    const float *res;          // optional, added to dx
    float *partial;            // [grid][Cw][Cn]
};

__device__ __forceinline__ f32x4 x3_mfma6_16(const bf16x8 (&a)[3], const bf16x8 (&b)[3], f32x4 acc)
{
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[2], b[0], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[0], b[2], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[1], b[1], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[1], b[0], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[0], b[1], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[0], b[0], acc, 0, 0, 0);
    return acc;
}

// eight values -> the three planes of an MFMA operand (value t in halfword t); p keeps the
// packed pairs (values 2t and 2t+1 of plane pl in p[t][pl])
__device__ __forceinline__ void x3_split8(const float (&v)[8], uint32_t (&p)[4][3], bf16x8 (&o)[3])
{
#pragma unroll
    for (int t = 0; t < 4; ++t)
        x3_split2(v[2 * t], v[2 * t + 1], p[t]);
#pragma unroll
    for (int pl = 0; pl < 3; ++pl) {
        const u32x4 q = {p[0][pl], p[1][pl], p[2][pl], p[3][pl]};
        o[pl] = __builtin_bit_cast(bf16x8, q);
    }
}

__device__ __forceinline__ void x3_wave_lds_fence()
{
    // a wavefront's LDS operations execute in order: only the compiler has to be held
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// NT: 16-channel tiles of the wide side (Cw <= 16*NT), even.
template <int NT, bool RES>
__global__ __launch_bounds__(256, 2) void bwd1x1_x3_kernel(X3Bwd1x1Args a)
{
    constexpr int KS = NT / 2;  // steps of 32 wide channels
    constexpr int PH = 40;      // halfwords per LDS row: 32 pixel positions + 8 (the 16-byte reads
                                // of 16 consecutive rows fall on distinct banks)
    constexpr int LD = 32 * PH; // one plane of a 32-channel step
    constexpr int LX = 16 * PH; // one plane of x
    constexpr int WAVE_HW = 3 * LD + 3 * LX;
    extern __shared__ uint16_t lds16[];
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, g = lane >> 4;
    uint16_t *Ld = lds16 + wv * WAVE_HW, *Lx = Ld + 3 * LD;
    const int Cn = a.Cn, Cw = a.Cw, HW = a.HW;

    // the BN-backward coefficients of the wide rows wait in LDS, {c0, c1, c2, -} per channel
    // (zero past the last row: de = 0); registers are what is scarce here
    f32x4 *Cl = reinterpret_cast<f32x4 *>(lds16 + 4 * WAVE_HW); // [16*NT]
    for (int c = threadIdx.x; c < 16 * NT; c += 256) {
        const int cc = c < Cw ? c : Cw - 1;
        const uint32_t m = c < Cw ? 0xffffffffu : 0u;
        Cl[c] = (f32x4){and_mask(a.c0[cc], m), and_mask(a.c1[cc], m), and_mask(a.c2[cc], m), 0.f};
    }
    // Element offsets are 32 bits (the host checks the tensors' sizes), so that a load is a
    // uniform base (tensor + t*HW, scalar registers) plus one vector register: the lane's eight
    // channels of step s start at row 32s + 8g, clamped to the last group of eight (Cw % 8 == 0;
    // groups past the end meet zero coefficients); rows 4g + v of x and dx, clamped likewise
    // (read, never stored).
    uint32_t vrow[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s)
        vrow[s] = (uint32_t)min(32 * s + 8 * g, Cw - 8) * (uint32_t)HW;
    uint32_t joff[4];
#pragma unroll
    for (int v = 0; v < 4; ++v)
        joff[v] = (uint32_t)(4 * g + v < Cn ? 4 * g + v : Cn - 1) * (uint32_t)HW;
    // W^T as the data gradient's A operand: row j = r, contraction = channels 32s + 8g .. +7
    bf16x8 wa[KS][3];
    {
        float wv8[KS][8];
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int c = 32 * s + 8 * g + t;
                const bool ok = c < Cw && r < Cn;
                wv8[s][t] = and_mask(a.w[ok ? (size_t)c * Cn + r : 0], ok ? 0xffffffffu : 0u);
            }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            uint32_t p[4][3];
            x3_split8(wv8[s], p, wa[s]);
        }
    }

    f32x4 acc[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
        acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const uint32_t vimg = (uint32_t)Cw * (uint32_t)HW, uimg = (uint32_t)Cn * (uint32_t)HW;
    const int cStep = 4 * (int)gridDim.x;
    int ch = 4 * (int)blockIdx.x + wv;
    // the lane's two pixels of chunk c (2r and 2r + 1: one image, HW being even): element
    // offsets in the wide tensors and in x / dx
    const auto locate = [&](int c, uint32_t &vb, uint32_t &ub, uint32_t &okm) {
        const uint32_t q = (uint32_t)c * 32u + 2u * (uint32_t)r;
        okm = q < a.Q ? 0xffffffffu : 0u;
        const uint32_t qs = q < a.Q ? q : 0u;
        const uint32_t n = fdiv(qs, a.divHW), pix = qs - n * (uint32_t)HW;
        vb = n * vimg + pix;
        ub = n * uimg + pix;
    };
    float vy[KS][2][8], ve[KS][2][8], xv[2][4];
    const auto fetch_step = [&](int s, uint32_t vb) {
        const uint32_t o = vb + vrow[s];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const float *py = a.dy + (size_t)t * HW, *pe = a.e + (size_t)t * HW; // uniform
            const f32x2 y2 = *reinterpret_cast<const f32x2 *>(py + o);
            const f32x2 e2 = *reinterpret_cast<const f32x2 *>(pe + o);
            vy[s][0][t] = y2[0];
            vy[s][1][t] = y2[1];
            ve[s][0][t] = e2[0];
            ve[s][1][t] = e2[1];
        }
    };
    const auto fetch_x = [&](uint32_t ub) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const f32x2 x2 = *reinterpret_cast<const f32x2 *>(a.x + ub + joff[v]);
            xv[0][v] = x2[0];
            xv[1][v] = x2[1];
        }
    };
    uint32_t vb, ub, okm;
    __syncthreads(); // Cl
    // (a wavefront without a chunk loads chunk 0 and never uses it)
    locate(ch < a.numChunks ? ch : 0, vb, ub, okm);
    fetch_x(ub);
#pragma unroll
    for (int s = 0; s < KS; ++s)
        fetch_step(s, vb);

    for (; ch < a.numChunks; ch += cStep) {
        // the next chunk (the last one re-reads itself: loads stay unconditional)
        const int nx = ch + cStep < a.numChunks ? ch + cStep : ch;
        uint32_t nvb, nub, nokm;
        locate(nx, nvb, nub, nokm);
        const uint32_t o0 = ub;
        const bool ook = okm != 0u;

        // x: the weight gradient's B operand (column j, contraction = pixels)
        {
            uint32_t w[4][3];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const uint32_t m = 4 * g + v < Cn ? okm : 0u;
                x3_split2(and_mask(xv[0][v], m), and_mask(xv[1][v], m), w[v]);
            }
            fetch_x(nub);
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    *reinterpret_cast<uint32_t *>(Lx + pl * LX + (4 * g + v) * PH + 2 * r) = w[v][pl];
        }
        x3_wave_lds_fence();
        bf16x8 bx[3];
#pragma unroll
        for (int pl = 0; pl < 3; ++pl)
            bx[pl] = x3_lds8(Lx + pl * LX + r * PH + 8 * g);

        f32x4 accd[2] = {(f32x4){0.f, 0.f, 0.f, 0.f}, (f32x4){0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            float d0[8], d1[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const f32x4 k = Cl[32 * s + 8 * g + t];
                d0[t] = and_mask(fmaf(k[0], vy[s][0][t], fmaf(k[1], ve[s][0][t], k[2])), okm);
                d1[t] = and_mask(fmaf(k[0], vy[s][1][t], fmaf(k[1], ve[s][1][t], k[2])), okm);
            }
            fetch_step(s, nvb);
            // data gradient: dx[j][pixel] += sum_c W[c][j] * de[c][pixel], straight from registers
            // (tile 0: the even pixels of the chunk, tile 1: the odd ones)
            uint32_t p0[4][3], p1[4][3];
            bf16x8 b0[3], b1[3];
            x3_split8(d0, p0, b0);
            x3_split8(d1, p1, b1);
            accd[0] = x3_mfma6_16(wa[s], b0, accd[0]);
            accd[1] = x3_mfma6_16(wa[s], b1, accd[1]);
            // transposed for the weight gradient: channel 8g + t, pixels 2r and 2r + 1
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
#pragma unroll
                for (int t2 = 0; t2 < 4; ++t2) {
                    const uint32_t lo = (p0[t2][pl] & 0xffffu) | (p1[t2][pl] << 16);
                    const uint32_t hi = (p0[t2][pl] >> 16) | (p1[t2][pl] & 0xffff0000u);
                    uint16_t *dst = Ld + pl * LD + (8 * g + 2 * t2) * PH + 2 * r;
                    *reinterpret_cast<uint32_t *>(dst) = lo;
                    *reinterpret_cast<uint32_t *>(dst + PH) = hi;
                }
            x3_wave_lds_fence();
            // weight gradient of the step's two 16-channel tiles
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2) {
                bf16x8 av[3];
#pragma unroll
                for (int pl = 0; pl < 3; ++pl)
                    av[pl] = x3_lds8(Ld + pl * LD + (16 * i2 + r) * PH + 8 * g);
                acc[2 * s + i2] = x3_mfma6_16(av, bx, acc[2 * s + i2]);
            }
            x3_wave_lds_fence(); // these reads before the next step's stores
        }
        f32x2 rs[4];
        if (RES) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                rs[v] = *reinterpret_cast<const f32x2 *>(a.res + o0 + joff[v]);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            f32x2 o = {accd[0][v], accd[1][v]};
            if (RES)
                o += rs[v];
            if (ook && 4 * g + v < Cn)
                *reinterpret_cast<f32x2 *>(a.dx + o0 + joff[v]) = o;
        }
        vb = nvb;
        ub = nub;
        okm = nokm;
    }
    // the four wavefronts' weight-gradient tiles, added in wavefront order
    __syncthreads();
    float *Rd = reinterpret_cast<float *>(Ld); // [16*NT][16] of this wavefront
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            Rd[(16 * i + 4 * g + v) * 16 + r] = acc[i][v];
    __syncthreads();
    float *dst = a.partial + (size_t)blockIdx.x * Cw * Cn;
    for (int el = threadIdx.x; el < 16 * NT * 16; el += 256) {
        const int c = el >> 4, j = el & 15;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            sum += reinterpret_cast<const float *>(lds16 + w * WAVE_HW)[el];
        if (c < Cw && j < Cn)
            dst[(size_t)c * Cn + j] = sum;
    }
}

bool bwd1x1_x3_supported(int Cw, int Cn, int HW)
{
    return Cn <= 16 && Cn < Cw && Cw <= 96 && Cw % 8 == 0 && HW % 2 == 0; // (pixel pairs)
}

// `splits` workgroups of four wavefronts; partial: [splits][Cw][Cn].
hipError_t launch_bwd1x1_x3(int N, int Cw, int Cn, int HW, const Operand &de, const void *xin,
                            const void *w, void *dx, const void *res, float *partial, int splits,
                            hipStream_t st)
{
    if (!bwd1x1_x3_supported(Cw, Cn, HW) || de.pro != PRO_BNBWD || splits < 1)
        return hipErrorInvalidValue;
    if ((long long)N * Cw * HW >= (1ll << 30)) // 32-bit byte offsets in the kernel
        return hipErrorInvalidValue;
    X3Bwd1x1Args a;
    a.Cn = Cn;
    a.Cw = Cw;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    a.numChunks = (int)((a.Q + 31u) / 32u);
    a.divHW = make_div((uint32_t)HW);
    a.x = (const float *)xin;
    a.dy = (const float *)de.p0;
    a.e = (const float *)de.p1;
    a.c0 = de.c0;
    a.c1 = de.c1;
    a.c2 = de.c2;
    a.w = (const float *)w;
    a.dx = (float *)dx;
    a.res = (const float *)res;
    a.partial = partial;
    const int nt = Cw <= 32 ? 2 : Cw <= 64 ? 4 : 6;
    // per wavefront three planes of a 32-channel step and of x (rows of 40 halfwords), and the
    // coefficient table
    const size_t lds = (size_t)4 * 3 * (32 + 16) * 40 * sizeof(uint16_t) + (size_t)16 * nt * 4 * sizeof(float);
#define MBK_CASE(NT_, RES_)                                                                       \
    if (nt == NT_ && (res != nullptr) == RES_) {                                                  \
        auto kern = bwd1x1_x3_kernel<NT_, RES_>;                                                  \
        const hipError_t e_ = hipFuncSetAttribute(                                                \
            (const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);            \
        if (e_ != hipSuccess)                                                                     \
            return e_;                                                                            \
        hipLaunchKernelGGL(kern, dim3((unsigned)splits), dim3(256), lds, st, a);                  \
        return hipGetLastError();                                                                 \
    }
    MBK_CASE(2, false)
    MBK_CASE(2, true)
    MBK_CASE(4, false)
    MBK_CASE(4, true)
    MBK_CASE(6, false)
    MBK_CASE(6, true)
#undef MBK_CASE
    return hipErrorInvalidValue;
}

// ---- 1x1 convolution with a short contraction: weights resident in LDS, a wavefront per chunk ----
// out[n][m][q] = sum_k W[m][k] * op(B)[n][k][q] for K <= 192 and many rows (the expansion conv,
// K = Cin, and the projection conv's data gradient, K = Cout, of the wide blocks).  In conv_x3
// every 64 x 64 output tile stages its own copy of the B operand (load, split into planes, LDS
// stores, two barriers per 32 values of k) and lasts 2-3 us per 32 values of k for 0.2 us of
// matrix-core time; with a short contraction the tile's prologue and epilogue are most of it.
// Here the roles are turned round:
//   - a workgroup owns a slab of 64 output rows; the slab's weights, all of K, are copied once
//     from the weight image into LDS (at most 72 KB) in the lane order of the MFMA's A operand,
//     so an operand is one 16-byte LDS read per lane and plane, conflict-free;
//   - a wavefront owns whole chunks of 32 pixels: lane (r, g) loads, for every 32 values of k,
//     the values k = 8g .. 8g+7 of its two pixels (2r and 2r+1 of the chunk when the plane size
//     is even: eight-byte loads, sixteen lanes cover a 128-byte line; r and 16+r otherwise),
//     which after the prologue and the split into planes ARE the B operands of
//     v_mfma_f32_16x16x32_bf16 (column = pixel, contraction = k): no LDS stores, no barrier in
//     the loop, and the operand is split once per pixel chunk and slab instead of once per tile;
//   - the next chunk's values of a k step are requested as soon as this chunk's have been
//     consumed; the accumulators (4 row tiles x 2 pixel tiles) are stored straight from
//     registers, eight bytes per lane, sixteen lanes to a 128-byte line;
//   - BN statistics of the output (EPI_STATS) are kept per lane over the wavefront's chunks and
//     reduced once at the end: lanes of a row, then the four wavefronts in order through LDS.
// Workgroup b: die = b % 8, then slab and chunk set, so that the workgroups of all slabs that
// read the same pixel chunks run on the same die and share its L2.
struct X3WArgs {
    int M, K, HW;
    uint32_t Q;
    int numChunks;
    FastDiv divHW;
    const uint16_t *img; // weight image in lane order
    X3Operand B;
    float *out;
    float *psum, *psq; // EPI_STATS: [M][NT]
    int NT;            // chunk sets (= statistics partials per row)
    int slabs;
};

template <int KS, bool PAIR, int PRO, int EPI>
__global__ __launch_bounds__(256, 2) void conv_xw_kernel(X3WArgs a)
{
    static_assert(PRO == PRO_NONE || PRO == PRO_BNBWD, "prologues of the short-contraction roles");
    static_assert(EPI == EPI_NONE || EPI == EPI_STATS, "epilogues of the short-contraction roles");
    constexpr int NP = PRO == PRO_BNBWD ? 2 : 1;
    constexpr int STEP_HW = 4 * 3 * 64 * 8; // halfwords of the slab per k step: 4 row tiles, 3 planes
    extern __shared__ uint16_t lds16[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;
    const int M = a.M, K = a.K, HW = a.HW;
    const int die = blockIdx.x & 7, bi = blockIdx.x >> 3;
    const int slab = bi % a.slabs, cs = (bi / a.slabs) * 8 + die;

    // the slab's weights: KS * 12 KB, copied as they lie in the image (requested here, parked in
    // LDS below, after the first chunk's values have been requested as well)
    u32x4 slabv[KS * 3];
    {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(a.img + (size_t)slab * KS * STEP_HW);
#pragma unroll
        for (int i = 0; i < KS * 3; ++i)
            slabv[i] = src[tid + 256 * i];
    }
    // BN-backward coefficients per contraction index, {c0, c1, c2, -} (zero past K)
    f32x4 *Cl = reinterpret_cast<f32x4 *>(lds16 + KS * STEP_HW); // [32*KS] (PRO_BNBWD)
    float *Rd = reinterpret_cast<float *>(lds16 + KS * STEP_HW); // [4][128]  (EPI_STATS, at the end)
    if (PRO == PRO_BNBWD) {
        for (int k = tid; k < 32 * KS; k += 256) {
            const int kk = k < K ? k : K - 1;
            const uint32_t m = k < K ? 0xffffffffu : 0u;
            Cl[k] = (f32x4){and_mask(a.B.c0[kk], m), and_mask(a.B.c1[kk], m), and_mask(a.B.c2[kk], m), 0.f};
        }
    }
    // the lane's eight contraction rows of step s start at row 32s + 8g, clamped to the last
    // group of eight (K % 8 == 0; the weight image is zero past K, the values read are finite)
    uint32_t vrow[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s)
        vrow[s] = (uint32_t)min(32 * s + 8 * g, K - 8) * (uint32_t)HW;
    const uint32_t mrow = (uint32_t)(64 * slab + 4 * g) * (uint32_t)HW; // output row 16i + v above it
    const uint32_t bimg = (uint32_t)K * (uint32_t)HW, oimg = (uint32_t)M * (uint32_t)HW;

    // pixel tile pt of chunk c: pixel 2r + pt (pairs) or r + 16 pt
    const auto locate = [&](int c, uint32_t (&bo)[2], uint32_t (&oo)[2], uint32_t (&okm)[2]) {
#pragma unroll
        for (int pt = 0; pt < (PAIR ? 1 : 2); ++pt) {
            const uint32_t q = (uint32_t)c * 32u + (PAIR ? 2u * (uint32_t)r : 16u * pt + (uint32_t)r);
            okm[pt] = q < a.Q ? 0xffffffffu : 0u;
            const uint32_t qs = q < a.Q ? q : 0u;
            const uint32_t n = fdiv(qs, a.divHW), pix = qs - n * (uint32_t)HW;
            bo[pt] = n * bimg + pix;
            oo[pt] = n * oimg + pix;
        }
        if (PAIR) {
            bo[1] = bo[0];
            oo[1] = oo[0];
            okm[1] = okm[0];
        }
    };
    float xv[NP][KS][2][8];
    const auto fetch_step = [&](int s, const uint32_t (&bo)[2]) {
        const uint32_t o0 = bo[0] + vrow[s], o1 = bo[1] + vrow[s];
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const float *pb = (p == 0 ? a.B.p0 : a.B.p1) + (size_t)t * HW; // uniform
                if (PAIR) {
                    const f32x2 v2 = *reinterpret_cast<const f32x2 *>(pb + o0);
                    xv[p][s][0][t] = v2[0];
                    xv[p][s][1][t] = v2[1];
                } else {
                    xv[p][s][0][t] = pb[o0];
                    xv[p][s][1][t] = pb[o1];
                }
            }
    };

    f32x4 acc[4][2];
    float s1[4][4], s2[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            s1[i][v] = s2[i][v] = 0.f;

    const int cStep = 4 * a.NT;
    int ch = 4 * cs + wv;
    uint32_t bo[2], oo[2], okm[2];
    locate(ch < a.numChunks ? ch : 0, bo, oo, okm);
#pragma unroll
    for (int s = 0; s < KS; ++s)
        fetch_step(s, bo);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < KS * 3; ++i)
        reinterpret_cast<u32x4 *>(lds16)[tid + 256 * i] = slabv[i];
    __syncthreads(); // the slab, Cl

    for (; ch < a.numChunks; ch += cStep) {
        const int nx = ch + cStep < a.numChunks ? ch + cStep : ch;
        uint32_t nbo[2], noo[2], nokm[2];
        locate(nx, nbo, noo, nokm);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            acc[i][0] = acc[i][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            float d0[8], d1[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                if (PRO == PRO_BNBWD) {
                    const f32x4 k = Cl[32 * s + 8 * g + t];
                    d0[t] = fmaf(k[0], xv[0][s][0][t], fmaf(k[1], xv[NP - 1][s][0][t], k[2]));
                    d1[t] = fmaf(k[0], xv[0][s][1][t], fmaf(k[1], xv[NP - 1][s][1][t], k[2]));
                } else {
                    d0[t] = xv[0][s][0][t];
                    d1[t] = xv[0][s][1][t];
                }
                d0[t] = and_mask(d0[t], okm[0]);
                d1[t] = and_mask(d1[t], okm[1]);
            }
            fetch_step(s, nbo);
            uint32_t p0[4][3], p1[4][3];
            bf16x8 b0[3], b1[3];
            x3_split8(d0, p0, b0);
            x3_split8(d1, p1, b1);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                bf16x8 av[3];
#pragma unroll
                for (int pl = 0; pl < 3; ++pl)
                    av[pl] = x3_lds8(lds16 + s * STEP_HW + ((i * 3 + pl) * 64 + lane) * 8);
                acc[i][0] = x3_mfma6_16(av, b0, acc[i][0]);
                acc[i][1] = x3_mfma6_16(av, b1, acc[i][1]);
            }
            // (one step at a time: the scheduler would otherwise split every step's operands
            // ahead of the first MFMA and run out of registers)
            __builtin_amdgcn_sched_barrier(0);
        }
        // rows 64 slab + 16i + 4g + v, the lane's two pixels
        const bool ok0 = okm[0] != 0u, ok1 = okm[1] != 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float *po = a.out + (size_t)(16 * i + v) * HW; // uniform
                const float x0 = acc[i][0][v], x1 = acc[i][1][v];
                const bool mok = 64 * slab + 16 * i + 4 * g + v < M;
                if (PAIR) {
                    if (ok0 && mok)
                        *reinterpret_cast<f32x2 *>(po + oo[0] + mrow) = (f32x2){x0, x1};
                } else {
                    if (ok0 && mok)
                        po[oo[0] + mrow] = x0;
                    if (ok1 && mok)
                        po[oo[1] + mrow] = x1;
                }
                if (EPI == EPI_STATS) { // (pixels past the end were masked to zero on the way in)
                    s1[i][v] += x0 + x1;
                    s2[i][v] = fmaf(x0, x0, fmaf(x1, x1, s2[i][v]));
                }
            }
#pragma unroll
        for (int pt = 0; pt < 2; ++pt) {
            bo[pt] = nbo[pt];
            oo[pt] = noo[pt];
            okm[pt] = nokm[pt];
        }
    }
    if (EPI == EPI_STATS) {
        // lanes of a row hold the same 16 channels: add them, then the wavefronts in order
        __syncthreads(); // (Rd lies over Cl)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float t1 = row16_sum(s1[i][v]), t2 = row16_sum(s2[i][v]);
                if (r == 0) {
                    Rd[wv * 128 + 16 * i + 4 * g + v] = t1;
                    Rd[wv * 128 + 64 + 16 * i + 4 * g + v] = t2;
                }
            }
        __syncthreads();
        if (tid < 128) {
            const int mm = 64 * slab + (tid & 63);
            const float t = (Rd[tid] + Rd[128 + tid]) + (Rd[256 + tid] + Rd[384 + tid]);
            if (mm < M)
                (tid < 64 ? a.psum : a.psq)[(size_t)mm * a.NT + cs] = t;
        }
    }
}

// Shapes and roles served: contraction of at most 192 (96 with the two-tensor prologue), a
// multiple of 8; at least one 64-row slab of output; fp32.  `nt`: chunk sets = statistics
// partials per row (a multiple of 8: one per die and round).
bool xw_conv_plan(int N, int M, int K, int HW, int pro, int epi, int *nt)
{
    const long long Q = (long long)N * HW;
    if (K % 8 != 0 || K < 32 || K > (pro == PRO_BNBWD ? 96 : 192) || M < 64 || M < K)
        return false;
    if ((pro != PRO_NONE && pro != PRO_BNBWD) || (epi != EPI_NONE && epi != EPI_STATS))
        return false;
    if (Q * M >= (1ll << 30) || Q * K >= (1ll << 30)) // 32-bit byte offsets in the kernel
        return false;
    const int slabs = (M + 63) / 64;
    const long long chunks = (Q + 31) / 32;
    // about two workgroups per CU in all, a multiple of 8 (one per die); of the counts that
    // need the same number of rounds over the chunk groups (four chunks, one per wavefront),
    // the smallest
    long long sets = (512 + slabs - 1) / slabs;
    sets = (sets + 7) / 8 * 8;
    const long long groups = (chunks + 3) / 4;
    if (sets > groups)
        sets = (groups + 7) / 8 * 8;
    const long long rounds = (groups + sets - 1) / sets;
    sets = ((groups + rounds - 1) / rounds + 7) / 8 * 8;
    *nt = (int)sets;
    return true;
}

hipError_t launch_xw_conv1x1(int N, int M, int K, int HW, const void *wimg, const Operand &B,
                             void *out, int epi, float *psum, float *psq, hipStream_t st)
{
    int nt;
    if (!xw_conv_plan(N, M, K, HW, B.pro, epi, &nt) || !wimg)
        return hipErrorInvalidValue;
    X3WArgs a;
    a.M = M;
    a.K = K;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    a.numChunks = (int)((a.Q + 31u) / 32u);
    a.divHW = make_div((uint32_t)HW);
    a.img = (const uint16_t *)wimg;
    a.B = to_x3(B);
    a.out = (float *)out;
    a.psum = psum;
    a.psq = psq;
    a.NT = nt;
    a.slabs = (M + 63) / 64;
    const int ks = (K + 31) / 32;
    const bool pair = HW % 2 == 0;
    const dim3 grid((unsigned)(a.slabs * nt));
    const size_t lds = (size_t)ks * 12288 + (B.pro == PRO_BNBWD ? std::max((size_t)ks * 512, (size_t)2048) : 2048);
#define MBK_CASE(KS_, PAIR_, PRO_, EPI_)                                                          \
    if (ks == KS_ && pair == PAIR_ && B.pro == PRO_ && epi == EPI_) {                             \
        auto kern = conv_xw_kernel<KS_, PAIR_, PRO_, EPI_>;                                       \
        const hipError_t e_ = hipFuncSetAttribute(                                                \
            (const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);            \
        if (e_ != hipSuccess)                                                                     \
            return e_;                                                                            \
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, a);                                    \
        return hipGetLastError();                                                                 \
    }
#define MBK_KS(KS_)                                                                               \
    MBK_CASE(KS_, true, PRO_NONE, EPI_STATS)                                                      \
    MBK_CASE(KS_, false, PRO_NONE, EPI_STATS)                                                     \
    MBK_CASE(KS_, true, PRO_NONE, EPI_NONE)                                                       \
    MBK_CASE(KS_, false, PRO_NONE, EPI_NONE)
    MBK_KS(1)
    MBK_KS(2)
    MBK_KS(3)
    MBK_KS(4)
    MBK_KS(5)
    MBK_KS(6)
#undef MBK_KS
#define MBK_KS(KS_)                                                                               \
    MBK_CASE(KS_, true, PRO_BNBWD, EPI_NONE)                                                      \
    MBK_CASE(KS_, false, PRO_BNBWD, EPI_NONE)                                                     \
    MBK_CASE(KS_, true, PRO_BNBWD, EPI_STATS)                                                     \
    MBK_CASE(KS_, false, PRO_BNBWD, EPI_STATS)
    MBK_KS(1)
    MBK_KS(2)
    MBK_KS(3)
    MBK_KS(4)
#undef MBK_KS
#undef MBK_CASE
    return hipErrorInvalidValue;
}

} // namespace mbk
