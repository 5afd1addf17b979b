// Host-side launchers of the gfx950 kernels (internal to libmbconv).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mbk {

// ---- operand of a 1x1 convolution with an elementwise prologue ------------------------
// The tensor is [N,C,HW] in the activation dtype.  What the GEMM consumes is
//   PRO_NONE         p0
//   PRO_BNSWISH_GATE swish(p0*c0[c]+c1[c]) * gate[n,c]       (Swish(BN(.)) times the SE gate)
//   PRO_BNBWD        c0[c]*p0 + c1[c]*p1 + c2[c]             (BN backward: p0 = dy, p1 = raw input)
enum { PRO_NONE = 0, PRO_BNSWISH_GATE = 1, PRO_BNBWD = 2 };
enum { EPI_NONE = 0, EPI_STATS = 1, EPI_RES = 2 };
constexpr int EPI_PARTIAL = 3; // internal: raw partial sums of a split contraction
// out = acc*scale[m] + shift[m] (+ res when res != NULL): a normalisation with fixed statistics
// folded into the epilogue (evaluation mode).  scale/shift travel in the psum/psq arguments of
// the internal launchers, read only.
constexpr int EPI_AFFINE = 4;

struct Operand {
    const void *p0 = nullptr;
    const void *p1 = nullptr;
    const float *c0 = nullptr, *c1 = nullptr, *c2 = nullptr;
    const float *gate = nullptr;
    int pro = PRO_NONE;
};

constexpr int kConvBQ = 128; // pixel columns per workgroup of the 1x1 conv kernel

inline int conv1x1_num_qtiles(int N, int HW) { return (int)(((long long)N * HW + kConvBQ - 1) / kConvBQ); }

// out[n,m,q] = sum_k A(m,k) * op(B)[n,k,q], A(m,k) = w[m*sAm + k*sAk] (dtype).
// epi: EPI_STATS writes partial sums of out and out^2 to psum/psq laid out
// [M][conv1x1_num_partials(...)]; EPI_RES adds res[n,m,q] before the store.
// sc_store (optional) receives the operand after its prologue (STORE policy).
// Long contractions with few output tiles are split over workgroups; `splitk_ws` then needs
// conv1x1_splitk_floats(...) floats (0 when the launch does not split).
// (`pro`, `epi`: the prologue and epilogue the launch will run with, where the caller knows
// them: some kernel families serve a shape only in certain roles; -1: not stated)
int conv1x1_num_partials(bool bf16, int N, int M, int K, int HW, bool stores_operand, int pro = -1,
                         int epi = -1);
// matrix-core instruction family of a launch: 1 fp32 MFMA, 2 bf16 MFMA on bf16 data, 3 bf16 MFMA
// on three-plane splits of fp32 data
int conv1x1_engine(bool bf16, int N, int M, int K, int HW, bool stores_operand, int pro = -1,
                   int epi = -1);
int wgrad1x1_engine(bool bf16, int Ma, int Mb, int N, int HW);
size_t conv1x1_splitk_floats(bool bf16, int N, int M, int K, int HW, bool stores_operand);
//
// fp32 convolutions of the wide blocks take their A operand from a weight image (bf16 planes in
// the order the kernel keeps them in LDS, see kernels_x3.hip): where
// conv1x1_uses_weight_image(...) says so, `wimg` must point to the image of this A (M rows, K
// contraction indices), x3_weight_image_bytes(M, K) bytes, written by launch_x3_prep beforehand;
// `w` is then not read.
bool conv1x1_uses_weight_image(bool bf16, int N, int M, int K, int HW, bool stores_operand,
                               int pro = -1, int epi = -1);
// 1: the kernel that serves this launch wants the image's tiles in lane order (launch_x3_prep)
int conv1x1_image_lane_order(bool bf16, int N, int M, int K, int HW, bool stores_operand, int pro,
                             int epi);
size_t x3_weight_image_bytes(int M, int K);
// Writes up to four images in one launch; image i is of A(m,k) = w[i][m*sm[i] + k*sk[i]], M[i] x K[i],
// its 64 x 32 tiles arranged as conv1x1_image_lane_order says (lane_order[i]).
hipError_t launch_x3_prep(int nsets, const float *const *w, const int *M, const int *K, const int *sm,
                          const int *sk, void *const *img, const int *lane_order, hipStream_t st);
hipError_t launch_conv1x1(bool bf16, int N, int M, int K, int HW, const void *w, int sAm, int sAk,
                          const Operand &B, void *out, int epi, const void *res, float *psum,
                          float *psq, void *sc_store, float *splitk_ws, hipStream_t st,
                          const void *wimg = nullptr);

// The same convolution with out = acc*scale[m] + shift[m] (+ res if non-null) as its epilogue.
// Returns hipErrorNotSupported (nothing launched) when the kernel family that serves this
// shape has no such epilogue; the caller then runs the convolution and the affine map as two
// steps.
hipError_t launch_conv1x1_affine(bool bf16, int N, int M, int K, int HW, const void *w, int sAm,
                                 int sAk, const Operand &B, void *out, const void *res,
                                 const float *scale, const float *shift, hipStream_t st,
                                 const void *wimg = nullptr);

// Weight gradient of a 1x1 conv: dW[a,b] = sum_{n,q} op(U)[n,a,q] * op(V)[n,b,q].
// `partial` needs wgrad_splits(...)*Ma*Mb floats.
int wgrad_splits(bool bf16, int Ma, int Mb, int N, int HW);
// With `defer` non-null the second stage (the sum over the splits) is not launched: it is
// described in *defer, and the caller launches it later (launch_reduce_splits2, together with
// another one); `partial` must stay untouched until then.
struct SplitReduce {
    const float *in; // [S][count]
    int S;
    size_t count;    // 0: no reduction
    float *out;      // [count]
};
hipError_t launch_wgrad1x1(bool bf16, int N, int Ma, int Mb, int HW, const Operand &U,
                           const Operand &V, float *partial, float *dW, SplitReduce *defer,
                           hipStream_t st);
hipError_t launch_reduce_splits2(const SplitReduce &a, const SplitReduce &b, hipStream_t st);
// Two independent weight gradients (A, B) in one launch, for the shapes wgrad1x1_pair_supported
// names; their second stages come back in *ra and *rb.  hipErrorNotSupported: nothing launched.
bool wgrad1x1_pair_supported(bool bf16, int N, int MaA, int MbA, int HWA, int MaB, int MbB, int HWB);
hipError_t launch_wgrad1x1_pair(bool bf16, int N, int MaA, int MbA, int HWA, const Operand &UA,
                                const Operand &VA, float *partialA, float *dWA, SplitReduce *ra,
                                int MaB, int MbB, int HWB, const Operand &UB, const Operand &VB,
                                float *partialB, float *dWB, SplitReduce *rb, hipStream_t st);

// Both gradients of a 1x1 convolution from Cn (narrow) to Cw (wide) channels in one pass over
// de, the gradient at its output (PRO_BNBWD operand, [N,Cw,HW]):
//   dx[n,j,q] = sum_c w[c*Cn+j] * de[n,c,q] (+ res[n,j,q]),   dW[c][j] = sum_{n,q} de[n,c,q] * x[n,j,q]
// bwd1x1_fused_plan tells whether the shape is covered (Cn <= 32, Cn < Cw <= 256, HW % 4 == 0) and
// how many splits of dW land in `partial` ([splits][Cw*Cn] floats, the count wgrad_splits gives);
// the caller sums them (launch_reduce_splits2).
// The mirror image for a convolution from Cw (wide) to Cn (narrow) channels, whose input sc is a
// PRO_BNSWISH_GATE or PRO_NONE operand [N,Cw,HW] and whose output gradient dp is PRO_BNBWD [N,Cn,HW]:
//   G[n,c,q] = sum_j w[j*Cw+c] * dp[n,j,q],   dW[j][c] = sum_{n,q} dp[n,j,q] * sc[n,c,q]
// `fin` (optional): dp's BN-backward coefficients are not read from dp.c0/c1/c2 but derived in
// the kernel from the per-plane partial sums, as launch_bn_bwd_finalize would (psb/psr: [Cn][NP],
// m elements per channel); workgroup 0 also stores dgamma, dbeta and the coefficient triple.
struct BnBwdFin {
    const float *psb, *psr, *gamma, *bn;
    float *dgamma, *dbeta, *coef;
    int NP;
    double m;
};
bool projbwd_fused_plan(int N, int Cw, int Cn, int HW, int *splits);
hipError_t launch_projbwd_fused(bool bf16, int N, int Cw, int Cn, int HW, const Operand &dp,
                                const Operand &sc, const void *w, void *G, float *partial,
                                int *splits_out, const BnBwdFin *fin, hipStream_t st);
bool bwd1x1_fused_plan(int N, int Cw, int Cn, int HW, int *splits);
// 0: not fused; else the mbconv_engine value of the kernel launch_bwd1x1_fused picks
int bwd1x1_fused_engine(bool bf16, int N, int Cw, int Cn, int HW);
hipError_t launch_bwd1x1_fused(bool bf16, int N, int Cw, int Cn, int HW, const Operand &de,
                               const void *xin, const void *w, void *dx, const void *res,
                               float *partial, int *splits_out, hipStream_t st);

// ---- batch-norm statistics ---------------------------------------------------------------
// Training-mode statistics that the consuming kernel finalises itself (no launch for the finalise
// step): the partial sums of the producer, and what the finalise step needs besides.
struct BnFin {
    const float *psum, *psq;   // [C][NP] partial sums and sums of squares
    const float *gamma, *beta; // [C]
    float *run_mean, *run_var; // [C] running statistics to update, or null
    float *bn_out;             // {scale, shift, mean, rstd}[C], written once per channel
    int NP;
    float eps, momentum;
    double inv_m;              // 1 / elements per channel
    double unbias;             // m/(m-1) (1 when m == 1): biased -> unbiased variance
};
inline BnFin make_bn_fin(const float *psum, const float *psq, const float *gamma, const float *beta,
                         float *run_mean, float *run_var, float *bn_out, int NP, float eps,
                         float momentum, double m)
{
    return {psum, psq, gamma, beta, run_mean, run_var, bn_out, NP, eps, momentum,
            1.0 / m, m > 1.0 ? m / (m - 1.0) : 1.0};
}

// psum/psq: [C][NP] partial sums.  Writes bn = {scale[C], shift[C], mean[C], rstd[C]} and
// updates running statistics (if non-null) with momentum.  If ones is non-null the same launch
// also sets ones[0..ones_count) to 1.
hipError_t launch_bn_finalize(int C, int NP, double m, const float *psum, const float *psq,
                              const float *gamma, const float *beta, float eps, float momentum,
                              float *run_mean, float *run_var, float *bn, hipStream_t st,
                              float *ones = nullptr, size_t ones_count = 0);

// Evaluation mode: the same blocks from running statistics, three normalisations per launch
// (C1 = 0 skips the first).
hipError_t launch_bn_eval_coef(int C1, const float *gamma1, const float *beta1, const float *rm1,
                               const float *rv1, float *bn1, int C2, const float *gamma2,
                               const float *beta2, const float *rm2, const float *rv2, float *bn2,
                               int C3, const float *gamma3, const float *beta3, const float *rm3,
                               const float *rv3, float *bn3, float eps, hipStream_t st);

// out[i] = value, i < count.
hipError_t launch_fill(float *out, float value, size_t count, hipStream_t st);

// Block without a squeeze-and-excitation stage (gate = 1, dz = 0): BN2's backward from the
// plane sums A1 = sum G*act'(y2), A2 = sum G*act'(y2)*dhat, both [N][C]:
//   dbeta = sum_n A1, dgamma = sum_n A2, coef as in launch_bn_bwd_finalize; dzs[N*C] is zeroed.
hipError_t launch_bn2_bwd_nose(int N, int C, double m, const float *A1, const float *A2,
                               const float *gamma, const float *bn, float *dgamma, float *dbeta,
                               float *coef, float *dzs, hipStream_t st);

// BN backward finalise from partial sums [C][NP] of dy (psb) and dy*xhat (psr):
//   dbeta = sum psb, dgamma = sum psr, and coef = {c0,c1,c2}[C] such that
//   dx = c0*dy + c1*raw + c2  equals  gamma*rstd*(dy - dbeta/m - xhat*dgamma/m).
hipError_t launch_bn_bwd_finalize(int C, int NP, double m, const float *psb, const float *psr,
                                  const float *gamma, const float *bn, float *dgamma,
                                  float *dbeta, float *coef, hipStream_t st);

// ---- depthwise chain ---------------------------------------------------------------------
struct DwShape {
    int N, C, H, W, Ho, Wo, k, s, p;
};
// Partial results per channel that launch_dw_fwd / launch_dw_bwd write (psum, psq, pdw, psb,
// psr are laid out [C][dw_num_partials]): one per image, or one per image range for the
// kernels that keep their accumulators across images.  `stores_a1`: the STORE policy is on.
int dw_num_partials(const DwShape &s, bool stores_a1);
size_t dw_fwd_lds_bytes(const DwShape &s);
size_t dw_bwd_lds_bytes(const DwShape &s);

// d = depthwise(swish(e*scale1+shift1)) (or depthwise(e) when bn1 == nullptr), plus per-plane
// partial sums of d and d^2 laid out [C][N].  a1_store (optional) receives swish(bn1(e)).
// With `fin` non-null (only when dw_fwd_finalizes_bn1 says so) the kernel derives bn1 from fin's
// partial sums and writes it to fin->bn_out; psum/psq must not overlap fin's partials.
bool dw_fwd_finalizes_bn1(const DwShape &s, bool stores_a1);
bool plane_finalize_pays(int HW); // launch_bn_apply: worth passing `fin` for planes of HW elements
hipError_t launch_dw_fwd(bool bf16, const DwShape &s, const void *e, const float *bn1,
                         const void *w_dw, void *d, float *psum, float *psq, void *a1_store,
                         const BnFin *fin, hipStream_t st);

// Per plane of d: z = mean swish(y2), s3 = sum swish'(y2), s4 = sum swish'(y2)*dhat.
hipError_t launch_pool(bool bf16, int N, int C, int HW, const void *d, const float *bn2, float *z,
                       float *s3, float *s4, hipStream_t st);

// SE excite: q = W1 z + b1, g = sigmoid(W2 swish(q) + b2).
hipError_t launch_se_fwd(int N, int C, int Cse, const float *z, const float *w1, const float *b1,
                         const float *w2, const float *b2, float *q, float *g, hipStream_t st);

// out = p*scale3+shift3 (+ x).
// With `fin` non-null the kernel derives bn3 from fin's partial sums and writes it to fin->bn_out.
hipError_t launch_bn_apply(bool bf16, int N, int C, int HW, const void *p, const float *bn3,
                           const void *res, void *out, const BnFin *fin, hipStream_t st);

// Per plane: sums of dy and dy*xhat with xhat = (raw-mean)*rstd, laid out [C][N].
hipError_t launch_plane_dot(bool bf16, int N, int C, int HW, const void *dy, const void *raw,
                            const float *bn, float *psb, float *psr, hipStream_t st);

// Per plane of (G, d): dg = sum G*a2, A1 = sum G*swish'(y2), A2 = sum G*swish'(y2)*dhat.
hipError_t launch_gate_sums(bool bf16, int N, int C, int HW, const void *G, const void *d,
                            const float *bn2, float *dg, float *A1, float *A2, hipStream_t st);

// SE backward.  Step 1 (one workgroup per image): dt, dq, dzs = dz/HW.
// Step 2: the four FC gradients, and BN2's dgamma/dbeta/coef from the plane sums.
struct SeBwdArgs {
    int N, C, Cse, HW;
    const float *z, *g, *q, *w1, *w2;
    const float *dg, *A1, *A2, *s3, *s4;
    const float *gamma2, *bn2;
    float *dt, *dq, *dzs;
    float *dw1, *db1, *dw2, *db2, *dgamma2, *dbeta2, *coef2;
};
hipError_t launch_se_bwd(const SeBwdArgs &a, hipStream_t st);

// The fused depthwise backward (per plane):
//   dy2 = (G*g + dzs)*swish'(y2);  dd = c0*dy2 + c1*d + c2  (BN2 backward)
//   dw partial[c][n][k*k] = sum dd * a1(shifted);  da1 = depthwise-transpose(dd)
//   with expansion: dy1 = da1*swish'(y1) -> dy1_out, partial sums of dy1 and dy1*e -> [C][N]
//   without:        dx = da1 (+ dout)            -> dx_out
struct DwBwdArgs {
    DwShape s;
    const void *G, *d, *e; // e is x when there is no expansion
    const float *g, *dzs, *bn2, *coef2, *bn1; // bn1 == nullptr: no expansion
    const void *w_dw;
    const void *a1_saved; // optional (STORE policy): swish(bn1(e)) saved by forward
    void *dy1_out;        // or dx when there is no expansion
    const void *res;      // residual dout (no-expansion case only)
    float *pdw, *psb, *psr;
};
hipError_t launch_dw_bwd(bool bf16, const DwBwdArgs &a, hipStream_t st);

// out[i] = sum_{s<S} in[s*count+i]  /  out[c*inner+i] = sum_{n<N} in[(c*N+n)*inner+i]
hipError_t launch_reduce_splits(const float *in, int S, size_t count, float *out, hipStream_t st);
hipError_t launch_reduce_planes(const float *in, int C, int N, int inner, float *out,
                                hipStream_t st);
// launch_reduce_planes(pdw, C, NP, inner, dw) and launch_bn_bwd_finalize(C, NP, m, psb, ...)
// in one launch (both consume the partial results of the fused depthwise backward).
hipError_t launch_dw_bwd_finalize(const float *pdw, int C, int NP, int inner, float *dw, double m,
                                  const float *psb, const float *psr, const float *gamma,
                                  const float *bn, float *dgamma, float *dbeta, float *coef,
                                  hipStream_t st);

} // namespace mbk
