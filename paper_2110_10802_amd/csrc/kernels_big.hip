// 1x1 convolutions and their weight gradients for the wide blocks (tens to a thousand
// channels on both sides), where the contraction is long enough to be bound by the matrix
// cores rather than by HBM.
//
// The batch is flattened: the GEMM column index is q = n*HW + pixel over all images, so small
// planes (14x14, 7x7) fill whole tiles.  A workgroup of four waves owns a (64*WT) x (64*WT) output
// tile, every wave a (32*WT) x (32*WT) block of v_mfma_f32_32x32x2_f32 accumulators; the
// contraction is consumed 16 (convolution) or 32 (weight gradient) at a time through two LDS
// buffers: the global loads of chunk i+1 are issued before the MFMAs of chunk i and land in LDS
// after them, so one barrier per chunk suffices.  The activation operand goes through its
// elementwise prologue on the way into LDS (Swish(BN(.))*gate, or the BN-backward expression),
// so these intermediates never exist in HBM (sections "Local Data Movement Reduction" and
// "Backpropagation and Data Movement").  Workgroups that share an activation tile are placed on
// the same XCD (blockIdx % 8) so the second read hits that XCD's L2.
#include "mbconv_dev.h"
#include "mbconv_launch.h"

namespace mbk {

typedef float float16v __attribute__((ext_vector_type(16)));

struct BigOperand {
    const void *p0, *p1;
    const float *c0, *c1, *c2, *gate;
};

// VEC consecutive elements of a tensor stored as T, widened to fp32
template <typename T, int VEC>
__device__ __forceinline__ void big_ld(const T *p, size_t i, float (&v)[VEC]);
template <>
__device__ __forceinline__ void big_ld<float, 4>(const float *p, size_t i, float (&v)[4])
{
    const float4 t = *reinterpret_cast<const float4 *>(p + i);
    v[0] = t.x;
    v[1] = t.y;
    v[2] = t.z;
    v[3] = t.w;
}
template <>
__device__ __forceinline__ void big_ld<float, 1>(const float *p, size_t i, float (&v)[1])
{
    v[0] = p[i];
}
template <>
__device__ __forceinline__ void big_ld<bf16_t, 4>(const bf16_t *p, size_t i, float (&v)[4])
{
    const uint2 t = *reinterpret_cast<const uint2 *>(&p[i]);
    v[0] = bf16_bits_to_float(t.x & 0xffffu);
    v[1] = bf16_bits_to_float(t.x >> 16);
    v[2] = bf16_bits_to_float(t.y & 0xffffu);
    v[3] = bf16_bits_to_float(t.y >> 16);
}
template <>
__device__ __forceinline__ void big_ld<bf16_t, 1>(const bf16_t *p, size_t i, float (&v)[1])
{
    v[0] = bf16_bits_to_float(p[i].bits);
}

// four consecutive elements stored as T
template <typename T>
__device__ __forceinline__ void big_st4(T *p, size_t i, const float (&v)[4]);
template <>
__device__ __forceinline__ void big_st4<float>(float *p, size_t i, const float (&v)[4])
{
    *reinterpret_cast<float4 *>(p + i) = make_float4(v[0], v[1], v[2], v[3]);
}
template <>
__device__ __forceinline__ void big_st4<bf16_t>(bf16_t *p, size_t i, const float (&v)[4])
{
    *reinterpret_cast<uint2 *>(&p[i]) =
        make_uint2(bf16_pack2(v[0], v[1]),
                   bf16_pack2(v[2], v[3]));
}

// Raw registers of one staged run of VEC elements of an operand row, with the row's
// prologue coefficients.  zero() makes apply() return 0 for every element.
template <int PRO, int VEC>
struct Staged {
    float v0[VEC];
    float v1[PRO == PRO_BNBWD ? VEC : 1];
    float k0, k1, k2; // BNBWD: c0,c1,c2; BNSWISH_GATE: scale, shift, gate

    __device__ __forceinline__ void zero()
    {
#pragma unroll
        for (int j = 0; j < VEC; ++j)
            v0[j] = 0.f;
        if (PRO == PRO_BNBWD) {
#pragma unroll
            for (int j = 0; j < VEC; ++j)
                v1[j] = 0.f;
        }
        k0 = k1 = k2 = 0.f;
    }
    template <typename T>
    __device__ __forceinline__ void load(const BigOperand &o, size_t idx)
    {
        big_ld<T, VEC>((const T *)o.p0, idx, v0);
        if constexpr (PRO == PRO_BNBWD)
            big_ld<T, VEC>((const T *)o.p1, idx, v1);
    }
    __device__ __forceinline__ float apply(int j) const
    {
        if (PRO == PRO_NONE)
            return v0[j];
        if (PRO == PRO_BNSWISH_GATE)
            return actf(fmaf(v0[j], k0, k1)) * k2;
        return fmaf(k0, v0[j], fmaf(k1, v1[PRO == PRO_BNBWD ? j : 0], k2));
    }
};

struct BigConvArgs {
    int M, K, HW;
    uint32_t Q; // N*HW
    FastDiv divHW;
    const void *w;
    int sAm, sAk;
    BigOperand B;
    void *out;
    const void *res;
    float *psum, *psq;
    int QT, MT; // tiles along q and m
    float *partial;     // EPI_PARTIAL: [splits][M][Q]
    int chunksPerSplit; // EPI_PARTIAL: chunks of BK of the contraction per blockIdx.y
};

// out[n,m,pix] = sum_k A(m,k) * op(B)[n,k,pix].  Requirements (checked by the host):
// K % 4 == 0, M % 4 == 0, HW % VEC == 0, one of sAm/sAk equal to 1.
template <typename T, int PRO, int EPI, int WM, int WP, int VEC, int D>
__global__ __launch_bounds__(256) void conv_big_kernel(BigConvArgs a)
{
    constexpr int BM = 64 * WM, BP = 64 * WP, BK = 16, KP = 1;
    constexpr int PA = BM + 4; // pitch = 4 mod 8: the transposing stores of A are 2-way at worst
    constexpr int NB = (VEC == 4 ? WP : 4 * WP) * KP; // staged runs of B per thread
    constexpr int BCOLS = BP / VEC;            // runs per row of the B tile
    constexpr int BROWS = 256 / BCOLS;         // rows staged per pass
    // One LDS block: the two operand buffers during the contraction, a 64 x 64 tile of results
    // (pitch CP) in the epilogue.
    constexpr int CP = 68;
    constexpr int OPER = 2 * BK * (PA + BP), TILE = 64 * CP;
    __shared__ __attribute__((aligned(16))) float smem[OPER > TILE ? OPER : TILE];
    __shared__ float red[2][BM][2];
    float(*As)[BK][PA] = reinterpret_cast<float(*)[BK][PA]>(smem);
    float(*Bs)[BK][BP] = reinterpret_cast<float(*)[BK][BP]>(smem + 2 * BK * PA);

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

    // ---- A staging ----
    float4 ra[D - 1][WM * KP];
    uint32_t raok[D - 1][WM * KP];
    // All staging loads are unconditional (indices clamped into the tensor, results masked
    // afterwards): straight-line code lets every load of a chunk be in flight at once, whereas
    // a branch per run makes the compiler wait for the previous run's data first.
    auto load_a = [&](int slot, int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < WM * KP; ++i) {
            float v[4];
            bool ok;
            if (kcontig) {
                const int m = m0 + (tid >> 2) + 64 * (i % WM), k = k0 + 16 * (i / WM) + 4 * (tid & 3);
                ok = m < a.M && k < a.K;
                big_ld<T, 4>((const T *)a.w, (size_t)min(m, a.M - 1) * a.sAm + min(k, a.K - 4), v);
            } else {
                const int m = m0 + 4 * (tid % (BM / 4)), k = k0 + tid / (BM / 4) + (1024 / BM) * i;
                ok = m < a.M && k < a.K;
                big_ld<T, 4>((const T *)a.w, (size_t)min(k, a.K - 1) * a.sAk + min(m, a.M - 4), v);
            }
            // the mask is applied when the run goes to LDS: touching the data here would make
            // the wavefront wait for the load it has just issued
            ra[slot][i] = make_float4(v[0], v[1], v[2], v[3]);
            raok[slot][i] = ok ? 0xffffffffu : 0u;
        }
    };
    auto store_a = [&](int slot, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < WM * KP; ++i) {
            const uint32_t mk = raok[slot][i];
            const float4 t = make_float4(and_mask(ra[slot][i].x, mk), and_mask(ra[slot][i].y, mk),
                                         and_mask(ra[slot][i].z, mk), and_mask(ra[slot][i].w, mk));
            if (kcontig) {
                const int m = (tid >> 2) + 64 * (i % WM), kk = 16 * (i / WM) + 4 * (tid & 3);
                As[buf][kk + 0][m] = t.x;
                As[buf][kk + 1][m] = t.y;
                As[buf][kk + 2][m] = t.z;
                As[buf][kk + 3][m] = t.w;
            } else {
                const int m = 4 * (tid % (BM / 4)), kk = tid / (BM / 4) + (1024 / BM) * i;
                *reinterpret_cast<float4 *>(&As[buf][kk][m]) = t;
            }
        }
    };

    // ---- B staging: this thread's pixel run is the same for every chunk ----
    const int bcol = tid % BCOLS, brow = tid / BCOLS;
    const uint32_t qb = q0 + (uint32_t)bcol * VEC;
    const bool bvalid = qb < a.Q;
    const uint32_t bn = bvalid ? fdiv(qb, a.divHW) : 0u; // an invalid column reads image 0, pixel 0
    const size_t bbase = (size_t)bn * a.K * a.HW + (bvalid ? qb - bn * (uint32_t)a.HW : 0u);
    Staged<PRO, VEC> rb[D - 1][NB];
    uint32_t rbok[D - 1][NB]; // all ones / zero: masking by AND keeps the staging code branch-free
    auto load_b = [&](int slot, int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int k = k0 + brow + BROWS * i;
            const int kc = min(k, a.K - 1);
            rbok[slot][i] = (bvalid && k < a.K) ? 0xffffffffu : 0u;
            rb[slot][i].template load<T>(a.B, bbase + (size_t)kc * a.HW);
            if (PRO == PRO_BNSWISH_GATE) {
                rb[slot][i].k0 = a.B.c0[kc];
                rb[slot][i].k1 = a.B.c1[kc];
                rb[slot][i].k2 = a.B.gate[(size_t)bn * a.K + kc];
            } else if (PRO == PRO_BNBWD) {
                rb[slot][i].k0 = a.B.c0[kc];
                rb[slot][i].k1 = a.B.c1[kc];
                rb[slot][i].k2 = a.B.c2[kc];
            }
        }
    };
    auto store_b = [&](int slot, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int kk = brow + BROWS * i;
            const uint32_t mk = rbok[slot][i];
            if (VEC == 4) {
                *reinterpret_cast<float4 *>(&Bs[buf][kk][4 * bcol]) =
                    make_float4(and_mask(rb[slot][i].apply(0), mk),
                                and_mask(rb[slot][i].apply(VEC == 4 ? 1 : 0), mk),
                                and_mask(rb[slot][i].apply(VEC == 4 ? 2 : 0), mk),
                                and_mask(rb[slot][i].apply(VEC == 4 ? 3 : 0), mk));
            } else {
                Bs[buf][kk][bcol] = and_mask(rb[slot][i].apply(0), mk);
            }
        }
    };

    float16v acc[WM][WP];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WP; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0.f;

    int cbeg = 0, cend = (a.K + BK - 1) / BK;
    if (EPI == EPI_PARTIAL) {
        cbeg = blockIdx.y * a.chunksPerSplit;
        cend = min(cbeg + a.chunksPerSplit, cend);
    }
    // Register ring of D-1 staged chunks: chunk j lives in slot (j - cbeg) % (D-1) from its load
    // until it is written to LDS, one iteration before it is consumed; its loads are issued D-1
    // iterations before that, so their latency is covered by D-2 iterations of MFMA work.
    // Every load and LDS store is unconditional (chunk indices clamped to the last chunk, whose
    // repeated copy is never consumed): with no branch between a load and its use the compiler's
    // wait counts stay exact, so the younger chunks really remain in flight while chunk cc+1 is
    // written to LDS.
    auto mfma_chunk = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float av[WM], bv[WP];
#pragma unroll
            for (int i = 0; i < WM; ++i)
                av[i] = As[buf][kk + (lane >> 5)][wm * 32 * WM + 32 * i + (lane & 31)];
#pragma unroll
            for (int j = 0; j < WP; ++j)
                bv[j] = Bs[buf][kk + (lane >> 5)][wp * 32 * WP + 32 * j + (lane & 31)];
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WP; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
    };
#pragma unroll
    for (int u = 0; u < D - 1; ++u) {
        const int cl = min(cbeg + u, cend - 1);
        load_a(u, cl * BK);
        load_b(u, cl * BK);
    }
    store_a(0, 0);
    store_b(0, 0);
    __syncthreads();
    auto step = [&](int u, int cc) __attribute__((always_inline)) {
        const int buf = (cc - cbeg) & 1;
        const int cl = min(cc + D - 1, cend - 1); // slot u is free: it went to LDS last iteration
        load_a(u, cl * BK);
        load_b(u, cl * BK);
        mfma_chunk(buf);
        store_a((u + 1) % (D - 1), buf ^ 1);
        store_b((u + 1) % (D - 1), buf ^ 1);
        __syncthreads();
    };
    // whole turns of the ring without any branch, then the remaining chunks
    const int turns = (cend - cbeg) / (D - 1), rest = (cend - cbeg) % (D - 1);
    int cc = cbeg;
    for (int g = 0; g < turns; ++g) {
#pragma unroll
        for (int u = 0; u < D - 1; ++u)
            step(u, cc + u);
        cc += D - 1;
    }
#pragma unroll
    for (int u = 0; u < D - 2; ++u)
        if (u < rest) // uniform over the workgroup
            step(u, cc + u);

    // ---- epilogue: register r of lane l is row 8*(r/4)+4*(l/32)+r%4, column l%32 ----
    if constexpr (VEC == 4 && WP == 1 && EPI != EPI_PARTIAL) {
        // Through LDS, 64 rows at a time: 16 lanes then own 64 consecutive pixels of one output
        // row, so the residual is read and the result written in 16-byte (fp32) or 8-byte
        // (bf16) pieces, and a row's statistics are a sum inside those 16 lanes.  (The last
        // chunk's barrier has passed: nobody reads the operand buffers any more.)
        float(*Ct)[CP] = reinterpret_cast<float(*)[CP]>(smem);
        const int pg = tid & 15;
        const uint32_t q = q0 + 4 * pg;
        const bool valid = q < a.Q;
        const uint32_t n = valid ? fdiv(q, a.divHW) : 0u;
        const uint32_t pix = valid ? q - n * (uint32_t)a.HW : 0u;
#pragma unroll
        for (int h = 0; h < WM; ++h) {
            if (h)
                __syncthreads();
            if (WM == 1 || wm == h) {
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        Ct[(WM == 1 ? wm * 32 : 32 * i) + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)]
                          [wp * 32 + (lane & 31)] = acc[i][0][r];
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = (tid >> 4) + 16 * i, m = m0 + 64 * h + row;
                const bool ok = valid && m < a.M;
                const float4 c = *reinterpret_cast<const float4 *>(&Ct[row][4 * pg]);
                float v[4] = {c.x, c.y, c.z, c.w};
                const size_t idx = ((size_t)n * a.M + min(m, a.M - 1)) * a.HW + pix;
                if (EPI == EPI_RES) {
                    float rr[4];
                    big_ld<T, 4>((const T *)a.res, idx, rr);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        v[j] += rr[j];
                }
                if (EPI == EPI_AFFINE) { // psum / psq carry the row's scale and shift
                    const float osc = a.psum[min(m, a.M - 1)], osh = a.psq[min(m, a.M - 1)];
                    float rr[4] = {0.f, 0.f, 0.f, 0.f};
                    if (a.res)
                        big_ld<T, 4>((const T *)a.res, idx, rr);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        v[j] = fmaf(v[j], osc, osh) + rr[j];
                }
                if (ok)
                    big_st4<T>((T *)a.out, idx, v);
                if (EPI == EPI_STATS) {
                    float s1 = 0.f, s2 = 0.f;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float sv = ok ? as_stored<T>(v[j]) : 0.f;
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
        }
        return;
    }
    float rs[WM][16], rq[WM][16];
    if (EPI == EPI_STATS) {
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                rs[i][r] = rq[i][r] = 0.f;
    }
#pragma unroll
    for (int j = 0; j < WP; ++j) {
        const uint32_t q = q0 + wp * 32 * WP + 32 * j + (lane & 31);
        const bool valid = q < a.Q;
        uint32_t n = 0, pix = 0;
        if (valid) {
            n = fdiv(q, a.divHW);
            pix = q - n * (uint32_t)a.HW;
        }
#pragma unroll
        for (int i = 0; i < WM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 32 * WM + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (EPI == EPI_PARTIAL) {
                    if (valid && m < a.M)
                        a.partial[((size_t)blockIdx.y * a.M + m) * a.Q + q] = acc[i][j][r];
                } else if (valid && m < a.M) {
                    float v = acc[i][j][r];
                    const size_t idx = ((size_t)n * a.M + m) * a.HW + pix;
                    if (EPI == EPI_RES)
                        v += ld<T>((const T *)a.res, idx);
                    st<T>((T *)a.out, idx, v);
                    if (EPI == EPI_STATS) {
                        const float sv = as_stored<T>(v);
                        rs[i][r] += sv;
                        rq[i][r] = fmaf(sv, sv, rq[i][r]);
                    }
                }
            }
        }
    }
    if (EPI == EPI_STATS) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float s = half_wave_sum_dpp(rs[i][r]);
                const float s2 = half_wave_sum_dpp(rq[i][r]);
                if ((lane & 31) == 0) {
                    const int row = wm * 32 * WM + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    red[0][row][wp] = s;
                    red[1][row][wp] = s2;
                }
            }
        }
        __syncthreads();
        if (tid < BM && m0 + tid < a.M) {
            a.psum[(size_t)(m0 + tid) * a.QT + qt] = red[0][tid][0] + red[0][tid][1];
            a.psq[(size_t)(m0 + tid) * a.QT + qt] = red[1][tid][0] + red[1][tid][1];
        }
    }
}

// Second stage of a split convolution: adds the partial tiles in a fixed order and applies the
// epilogue.  A workgroup owns 1024 consecutive q of one output channel.
template <typename T, int EPI>
__global__ __launch_bounds__(256) void splitk_finish_kernel(const float *__restrict__ partial, int S,
                                                            int M, uint32_t Q, FastDiv divHW, int HW,
                                                            T *out, const T *res, float *psum,
                                                            float *psq, int NT)
{
    __shared__ float red[2][4];
    const int m = blockIdx.y, tid = threadIdx.x;
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t q = blockIdx.x * 1024u + 256u * i + tid;
        if (q < Q) {
            // four independent running sums keep the loads of a round in flight together
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
                v += ld<T>(res, idx);
            st<T>(out, idx, v);
            if (EPI == EPI_STATS) {
                const float sv = as_stored<T>(v);
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

static BigOperand to_big(const Operand &o)
{
    BigOperand d;
    d.p0 = o.p0;
    d.p1 = o.p1;
    d.c0 = o.c0;
    d.c1 = o.c1;
    d.c2 = o.c2;
    d.gate = o.gate;
    return d;
}

// 128 rows per tile when that pads the channel count no further than 64 would
static int big_rows(int M) { return ((M + 127) / 128) * 128 == ((M + 63) / 64) * 64 ? 2 : 1; }

// Tile choice; `wt` packs the row and column factors as 4*WM + WP.  When the tiles are too few to fill
// the chip and the contraction is long, it is split `splits` ways (each at least four chunks of
// 16) and a second kernel adds the partial tiles; `qtiles` is then that kernel's count of
// 1024-pixel groups.
bool big_conv_plan(int N, int M, int K, int HW, int *wt, int *qtiles, int *splits)
{
    const long long Q = (long long)N * HW;
    if (K % 4 != 0 || M % 4 != 0 || Q >= (1ll << 31) || K < 16)
        return false;
    // measured: 64-column tiles are never slower than 128-column ones (more workgroups in
    // flight matter more than operand reuse); 128 rows pay only for very wide outputs
    const int wm = M >= 512 ? big_rows(M) : 1;
    const int wp = 1;
    *wt = 4 * wm + wp;
    *qtiles = (int)((Q + 64 * wp - 1) / (64 * wp));
    *splits = 1;
    const long long tiles = (long long)*qtiles * ((M + 64 * wm - 1) / (64 * wm));
    const int chunks = (K + 15) / 16;
    if (wp == 1 && tiles < 384 && chunks >= 16) {
        long long s = (768 + tiles - 1) / tiles;
        if (s > chunks / 4)
            s = chunks / 4;
        if (s > 16)
            s = 16;
        const int per = (int)((chunks + s - 1) / s);
        *splits = (chunks + per - 1) / per;
        if (*splits > 1)
            *qtiles = (int)((Q + 1023) / 1024);
    }
    return true;
}

#ifndef MBK_BIG_D
#define MBK_BIG_D 3
#endif
template <typename T, int WM, int WP, int VEC, int D = MBK_BIG_D>
static hipError_t big_conv_dispatch(const BigConvArgs &a, int pro, int epi, dim3 grid, hipStream_t st)
{
#define MBK_CASE(P, E)                                                                            \
    if (pro == P && epi == E) {                                                                   \
        hipLaunchKernelGGL((conv_big_kernel<T, P, E, WM, WP, VEC, D>), grid, dim3(256), 0, st,    \
                           a);                                                                    \
        return hipGetLastError();                                                                 \
    }
    MBK_CASE(PRO_NONE, EPI_STATS)
    MBK_CASE(PRO_BNSWISH_GATE, EPI_STATS)
    MBK_CASE(PRO_BNBWD, EPI_NONE)
    MBK_CASE(PRO_BNBWD, EPI_RES)
    if constexpr (WP == 1 && VEC == 4) {
        MBK_CASE(PRO_BNSWISH_GATE, EPI_AFFINE)
    }
    if constexpr (WP == 1) {
        MBK_CASE(PRO_NONE, EPI_PARTIAL)
        MBK_CASE(PRO_BNSWISH_GATE, EPI_PARTIAL)
        MBK_CASE(PRO_BNBWD, EPI_PARTIAL)
    }
#undef MBK_CASE
    return hipErrorInvalidValue;
}

template <typename T>
static hipError_t splitk_finish(const float *partial, int S, int M, uint32_t Q, int HW, void *out,
                                const void *res, int epi, float *psum, float *psq, int NT,
                                hipStream_t st)
{
    dim3 grid((unsigned)NT, (unsigned)M);
    const FastDiv dv = make_div((uint32_t)HW);
#define MBK_CASE(E)                                                                               \
    if (epi == E) {                                                                               \
        hipLaunchKernelGGL((splitk_finish_kernel<T, E>), grid, dim3(256), 0, st, partial, S, M, Q, \
                           dv, HW, (T *)out, (const T *)res, psum, psq, NT);                      \
        return hipGetLastError();                                                                 \
    }
    MBK_CASE(EPI_NONE)
    MBK_CASE(EPI_STATS)
    MBK_CASE(EPI_RES)
#undef MBK_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_splitk_finish_f32(const float *partial, int S, int M, uint32_t Q, int HW, void *out,
                                    const void *res, int epi, float *psum, float *psq, int NT,
                                    hipStream_t st)
{
    return splitk_finish<float>(partial, S, M, Q, HW, out, res, epi, psum, psq, NT, st);
}

size_t big_conv_splitk_floats(int N, int M, int K, int HW)
{
    int wt, qtiles, splits;
    if (!big_conv_plan(N, M, K, HW, &wt, &qtiles, &splits) || splits == 1)
        return 0;
    return (size_t)splits * M * N * HW;
}

hipError_t launch_big_conv1x1(bool bf16, int N, int M, int K, int HW, const void *w, int sAm,
                              int sAk, const Operand &B, void *out, int epi, const void *res,
                              float *psum, float *psq, float *splitk_ws, hipStream_t st)
{
    int wt, qtiles, splits;
    if (!big_conv_plan(N, M, K, HW, &wt, &qtiles, &splits) || (sAm != 1 && sAk != 1))
        return hipErrorInvalidValue;
    if (splits > 1 && !splitk_ws)
        return hipErrorInvalidValue;
    BigConvArgs a;
    a.M = M;
    a.K = K;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    a.divHW = make_div((uint32_t)HW);
    a.w = w;
    a.sAm = sAm;
    a.sAk = sAk;
    a.B = to_big(B);
    a.out = out;
    a.res = res;
    a.psum = psum;
    a.psq = psq;
    const int wm = wt >> 2, wp = wt & 3;
    a.QT = (int)((a.Q + 64u * wp - 1) / (64u * wp));
    a.MT = (M + 64 * wm - 1) / (64 * wm);
    a.partial = splitk_ws;
    const int chunks = (K + 15) / 16;
    a.chunksPerSplit = (chunks + splits - 1) / splits;
    dim3 grid((unsigned)(((a.QT + 7) / 8) * 8 * a.MT), (unsigned)splits);
    const bool v4 = HW % 4 == 0;
    if (!v4 && wp != 1)
        return hipErrorInvalidValue;
    const int user_epi = epi;
    if (splits > 1)
        epi = EPI_PARTIAL;
#define MBK_GO(TT)                                                                                \
    (!v4 ? (wm == 2 ? big_conv_dispatch<TT, 2, 1, 1>(a, B.pro, epi, grid, st)                     \
                    : big_conv_dispatch<TT, 1, 1, 1>(a, B.pro, epi, grid, st))                    \
         : (wm == 2 ? big_conv_dispatch<TT, 2, 1, 4>(a, B.pro, epi, grid, st)                     \
                    : big_conv_dispatch<TT, 1, 1, 4>(a, B.pro, epi, grid, st)))
    if (wp != 1)
        return hipErrorInvalidValue;
    const hipError_t e = bf16 ? MBK_GO(bf16_t) : MBK_GO(float);
#undef MBK_GO
    if (e != hipSuccess || splits == 1)
        return e;
    return bf16 ? splitk_finish<bf16_t>(splitk_ws, splits, M, a.Q, HW, out, res, user_epi, psum,
                                        psq, qtiles, st)
                : splitk_finish<float>(splitk_ws, splits, M, a.Q, HW, out, res, user_epi, psum, psq,
                                       qtiles, st);
}

// ---- weight gradient -------------------------------------------------------------------
// dW[a,b] = sum_q op(U)[a,q] * op(V)[b,q]: both operands are pixel-contiguous in memory and
// the matrix cores want the channel index across lanes, so both tiles are transposed on their
// way into LDS ([q][channel], pitch = 2 mod 8 keeps the scalar stores 2-way at worst).  The
// contraction is split over blockIdx.z; each split writes its own partial tile and a
// fixed-order second stage adds them (no atomics: the map-fission step of section "Guided
// Optimization Case Study: EfficientNet").

struct BigWgradArgs {
    int Ma, Mb, HW;
    uint32_t Q;
    int chunksPerSplit; // chunks of 32 pixels
    FastDiv divHW;
    BigOperand U, V;
    float *partial;
};

// (bx, by, bz: tile of U rows, tile of V rows, split; Us, Vs: the LDS buffers)
template <typename T, int PROU, int PROV, int WA, int WB, int VEC>
__device__ __forceinline__ void wgrad_big_body(const BigWgradArgs &a, int bx, int by, int bz,
                                               float (*Us)[32][64 * WA + 2], float (*Vs)[32][64 * WB + 2])
{
    constexpr int BA = 64 * WA, BB = 64 * WB, BQ = 32;
    constexpr int QCOLS = BQ / VEC;     // runs per operand row
    constexpr int RROWS = 256 / QCOLS;  // rows staged per pass
    constexpr int NRU = BA / RROWS, NRV = BB / RROWS; // runs per thread of U and of V
    // two LDS buffers, except for the 128x128 tile, where two would exceed 64 KiB
    constexpr int NBUF = (WA == 2 && WB == 2) ? 1 : 2;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wa = wave >> 1, wb = wave & 1;
    const int a0 = bx * BA, b0 = by * BB;
    const int numChunks = (int)((a.Q + BQ - 1) / BQ);
    const int cbeg = bz * a.chunksPerSplit;
    const int cend = min(cbeg + a.chunksPerSplit, numChunks);

    const int qcol = tid % QCOLS, rrow = tid / QCOLS;
    Staged<PROU, VEC> ru[NRU];
    Staged<PROV, VEC> rv[NRV];
    // per-row coefficients do not depend on the chunk (rows past the end keep zeros, which
    // make apply() return 0 for zero data)
#pragma unroll
    for (int i = 0; i < NRU; ++i) {
        const int ra = a0 + rrow + RROWS * i;
        ru[i].zero();
        if (PROU != PRO_NONE && ra < a.Ma) {
            ru[i].k0 = a.U.c0[ra];
            ru[i].k1 = a.U.c1[ra];
            if (PROU == PRO_BNBWD)
                ru[i].k2 = a.U.c2[ra];
        }
    }
#pragma unroll
    for (int i = 0; i < NRV; ++i) {
        const int rb = b0 + rrow + RROWS * i;
        rv[i].zero();
        if (PROV != PRO_NONE && rb < a.Mb) {
            rv[i].k0 = a.V.c0[rb];
            rv[i].k1 = a.V.c1[rb];
            if (PROV == PRO_BNBWD)
                rv[i].k2 = a.V.c2[rb];
        }
    }
    // Unconditional loads with clamped indices (see conv_big_kernel): rows past the end read
    // the last row, a run past the end reads pixel 0; both are zeroed by an AND mask on their
    // way into LDS, so there is no branch between a load and its use.
    uint32_t umask[NRU], vmask[NRV], qmask = 0u;
#pragma unroll
    for (int i = 0; i < NRU; ++i)
        umask[i] = a0 + rrow + RROWS * i < a.Ma ? 0xffffffffu : 0u;
#pragma unroll
    for (int i = 0; i < NRV; ++i)
        vmask[i] = b0 + rrow + RROWS * i < a.Mb ? 0xffffffffu : 0u;
    auto load = [&](int chunk) __attribute__((always_inline)) {
        const uint32_t q = (uint32_t)chunk * BQ + (uint32_t)qcol * VEC;
        const bool valid = q < a.Q;
        qmask = valid ? 0xffffffffu : 0u;
        const uint32_t qc = valid ? q : 0u;
        const uint32_t n = fdiv(qc, a.divHW);
        const uint32_t pix = qc - n * (uint32_t)a.HW;
#pragma unroll
        for (int i = 0; i < NRU; ++i) {
            const int ra = min(a0 + rrow + RROWS * i, a.Ma - 1);
            ru[i].template load<T>(a.U, ((size_t)n * a.Ma + ra) * a.HW + pix);
            if (PROU == PRO_BNSWISH_GATE)
                ru[i].k2 = a.U.gate[(size_t)n * a.Ma + ra];
        }
#pragma unroll
        for (int i = 0; i < NRV; ++i) {
            const int rb = min(b0 + rrow + RROWS * i, a.Mb - 1);
            rv[i].template load<T>(a.V, ((size_t)n * a.Mb + rb) * a.HW + pix);
            if (PROV == PRO_BNSWISH_GATE)
                rv[i].k2 = a.V.gate[(size_t)n * a.Mb + rb];
        }
    };
    auto store = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NRU; ++i) {
#pragma unroll
            for (int j = 0; j < VEC; ++j)
                Us[buf][qcol * VEC + j][rrow + RROWS * i] = and_mask(ru[i].apply(j), qmask & umask[i]);
        }
#pragma unroll
        for (int i = 0; i < NRV; ++i) {
#pragma unroll
            for (int j = 0; j < VEC; ++j)
                Vs[buf][qcol * VEC + j][rrow + RROWS * i] = and_mask(rv[i].apply(j), qmask & vmask[i]);
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
        load(cbeg);
        store(0);
        __syncthreads();
        for (int c = cbeg; c < cend; ++c) {
            const int buf = NBUF == 2 ? (c - cbeg) & 1 : 0;
            load(min(c + 1, cend - 1)); // the repeated last chunk is stored but never consumed
#pragma unroll
            for (int kk = 0; kk < BQ; kk += 2) {
                float av[WA], bv[WB];
#pragma unroll
                for (int i = 0; i < WA; ++i)
                    av[i] = Us[buf][kk + (lane >> 5)][wa * 32 * WA + 32 * i + (lane & 31)];
#pragma unroll
                for (int j = 0; j < WB; ++j)
                    bv[j] = Vs[buf][kk + (lane >> 5)][wb * 32 * WB + 32 * j + (lane & 31)];
#pragma unroll
                for (int i = 0; i < WA; ++i)
#pragma unroll
                    for (int j = 0; j < WB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
            }
            if (NBUF == 1)
                __syncthreads();
            store(NBUF == 2 ? buf ^ 1 : 0);
            __syncthreads();
        }
    }
    float *dst = a.partial + (size_t)bz * a.Ma * a.Mb;
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

template <typename T, int PROU, int PROV, int WA, int WB, int VEC>
__global__ __launch_bounds__(256) void wgrad_big_kernel(BigWgradArgs a)
{
    constexpr int NBUF = (WA == 2 && WB == 2) ? 1 : 2;
    __shared__ __attribute__((aligned(16))) float Us[NBUF][32][64 * WA + 2];
    __shared__ __attribute__((aligned(16))) float Vs[NBUF][32][64 * WB + 2];
    wgrad_big_body<T, PROU, PROV, WA, WB, VEC>(a, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, Us, Vs);
}

// Two weight gradients of one block in one launch (64 x 64 tiles, no run vectorisation: the 7x7
// stages): the launches are a few hundred workgroups each and bound by the latency of their own
// load-stage-multiply chain, so together they fill the wavefront slots either leaves empty.
// The first gridA workgroups work on `a` (projection conv: dp x gated activation), the others on
// `b` (expansion conv: de x block input); tiles and splits are decoded from the linear index.
template <typename T>
__global__ __launch_bounds__(256) void wgrad_big_pair_kernel(BigWgradArgs a, BigWgradArgs b, int gridA)
{
    __shared__ __attribute__((aligned(16))) float Us[2][32][66];
    __shared__ __attribute__((aligned(16))) float Vs[2][32][66];
    if ((int)blockIdx.x < gridA) { // uniform over the workgroup
        const int i = (int)blockIdx.x, ta = (a.Ma + 63) / 64, tb = (a.Mb + 63) / 64;
        wgrad_big_body<T, PRO_BNBWD, PRO_BNSWISH_GATE, 1, 1, 1>(a, i % ta, (i / ta) % tb, i / (ta * tb), Us, Vs);
    } else {
        const int i = (int)blockIdx.x - gridA, ta = (b.Ma + 63) / 64, tb = (b.Mb + 63) / 64;
        wgrad_big_body<T, PRO_BNBWD, PRO_NONE, 1, 1, 1>(b, i % ta, (i / ta) % tb, i / (ta * tb), Us, Vs);
    }
}

// `wt` packs the tile factors as 4*WA + WB.
bool big_wgrad_plan(int Ma, int Mb, int N, int HW, int *wt, int *splits)
{
    const long long Q = (long long)N * HW;
    if (Q >= (1ll << 31))
        return false;
    // measured: 64x64 tiles with many contraction splits beat larger tiles on every shape of
    // the late EfficientNet stages (workgroups in flight hide the staging latency)
    const int wa = 1, wb = 1;
    *wt = 4 * wa + wb;
    const long long tiles = (long long)((Ma + 63) / 64) * ((Mb + 63) / 64);
    const long long chunks = (Q + 31) / 32;
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

template <typename T, int WA, int WB, int VEC>
static hipError_t big_wgrad_dispatch(const BigWgradArgs &a, int pu, int pv, dim3 grid, hipStream_t st)
{
#define MBK_CASE(PU, PV)                                                                          \
    if (pu == PU && pv == PV) {                                                                   \
        hipLaunchKernelGGL((wgrad_big_kernel<T, PU, PV, WA, WB, VEC>), grid, dim3(256), 0, st, a); \
        return hipGetLastError();                                                                 \
    }
    MBK_CASE(PRO_BNBWD, PRO_NONE)
    MBK_CASE(PRO_BNBWD, PRO_BNSWISH_GATE)
#undef MBK_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_big_wgrad(bool bf16, int N, int Ma, int Mb, int HW, const Operand &U,
                            const Operand &V, float *partial, int *splits_out, hipStream_t st)
{
    int wt, splits;
    if (!big_wgrad_plan(Ma, Mb, N, HW, &wt, &splits))
        return hipErrorInvalidValue;
    const int wa = wt >> 2, wb = wt & 3;
    BigWgradArgs a;
    a.Ma = Ma;
    a.Mb = Mb;
    a.HW = HW;
    a.Q = (uint32_t)((long long)N * HW);
    const int chunks = (int)((a.Q + 31u) / 32u);
    a.chunksPerSplit = (chunks + splits - 1) / splits;
    a.divHW = make_div((uint32_t)HW);
    a.U = to_big(U);
    a.V = to_big(V);
    a.partial = partial;
    *splits_out = splits;
    dim3 grid((unsigned)((Ma + 64 * wa - 1) / (64 * wa)), (unsigned)((Mb + 64 * wb - 1) / (64 * wb)),
              (unsigned)splits);
    const bool v4 = HW % 4 == 0;
#define MBK_GO(TT)                                                                                \
    (!v4 ? big_wgrad_dispatch<TT, 1, 1, 1>(a, U.pro, V.pro, grid, st)                             \
         : big_wgrad_dispatch<TT, 1, 1, 4>(a, U.pro, V.pro, grid, st))
    if (wa != 1 || wb != 1)
        return hipErrorInvalidValue;
    return bf16 ? MBK_GO(bf16_t) : MBK_GO(float);
#undef MBK_GO
}

// The pair of launch_big_wgrad calls (A: U = BN-backward operand, V = gated activation; B: U =
// BN-backward operand, V = plain) in one launch; hipErrorNotSupported (nothing launched) for
// other operand kinds, tile shapes or plane sizes that are a multiple of four.
hipError_t launch_big_wgrad_pair(bool bf16, int N, int MaA, int MbA, int HWA, const Operand &UA,
                                 const Operand &VA, float *partialA, int *splitsA, int MaB, int MbB,
                                 int HWB, const Operand &UB, const Operand &VB, float *partialB,
                                 int *splitsB, hipStream_t st)
{
    int wta, wtb, sa, sb;
    if (!big_wgrad_plan(MaA, MbA, N, HWA, &wta, &sa) || !big_wgrad_plan(MaB, MbB, N, HWB, &wtb, &sb))
        return hipErrorNotSupported;
    if (wta != 5 || wtb != 5 || HWA % 4 == 0 || HWB % 4 == 0 || UA.pro != PRO_BNBWD ||
        VA.pro != PRO_BNSWISH_GATE || UB.pro != PRO_BNBWD || VB.pro != PRO_NONE)
        return hipErrorNotSupported;
    const auto fill = [N](BigWgradArgs &a, int Ma, int Mb, int HW, const Operand &U, const Operand &V,
                          float *partial, int splits) {
        a.Ma = Ma;
        a.Mb = Mb;
        a.HW = HW;
        a.Q = (uint32_t)((long long)N * HW);
        const int chunks = (int)((a.Q + 31u) / 32u);
        a.chunksPerSplit = (chunks + splits - 1) / splits;
        a.divHW = make_div((uint32_t)HW);
        a.U = to_big(U);
        a.V = to_big(V);
        a.partial = partial;
        return ((Ma + 63) / 64) * ((Mb + 63) / 64) * splits;
    };
    BigWgradArgs a, b;
    const int ga = fill(a, MaA, MbA, HWA, UA, VA, partialA, sa);
    const int gb = fill(b, MaB, MbB, HWB, UB, VB, partialB, sb);
    *splitsA = sa;
    *splitsB = sb;
    if (bf16)
        hipLaunchKernelGGL(wgrad_big_pair_kernel<bf16_t>, dim3((unsigned)(ga + gb)), dim3(256), 0, st, a, b, ga);
    else
        hipLaunchKernelGGL(wgrad_big_pair_kernel<float>, dim3((unsigned)(ga + gb)), dim3(256), 0, st, a, b, ga);
    return hipGetLastError();
}

} // namespace mbk
