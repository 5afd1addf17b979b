// C ABI of libmbconv: argument validation, workspace layout and the launch sequence of
// one MBConv training step.  See include/mbconv.h for the contract.
#include "../../include/mbconv.h"
#include "mbconv_launch.h"

#include <algorithm>
#include <cstdint>

// The launch sequence below is compiled twice: once as is (namespace mbk, Swish) and once with
// -Dmbk=mbk_r6 -DMBK_ACT_RELU6 (ReLU6 kernels); the C entry points exist in the first build
// only and pick the namespace by desc->activation.
namespace mbk {

namespace {

constexpr size_t kAlign = 256;
constexpr size_t kAbsent = SIZE_MAX;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Plan {
    int N, Cin, H, W, Cexp, Cse, Cout, k, s, p, Ho, Wo;
    bool expand, res, bf16, store, se;
    size_t esz;
    size_t nX, nE, nD, nP;
    int HW, HWo;
    // saved workspace (byte offsets)
    size_t o_e, o_d, o_p, o_bn1, o_bn2, o_bn3, o_z, o_g, o_q, o_s3, o_s4, o_a1, o_sc, saved_bytes;
    // weight images of the four 1x1 convolutions (kAbsent where the kernel family that serves
    // the shape reads the weights themselves): expansion conv, projection conv, projection data
    // gradient, expansion data gradient; written by forward, read again by backward
    size_t o_wimg[4];
    int wimg_lane_order[4]; // how the kernel that reads image i wants its tiles arranged
    // scratch workspace (byte offsets)
    size_t o_part;  // partial sums: 2 arrays of part_floats
    size_t o_wg2;   // projection weight gradient's partials while their reduction is deferred
    size_t o_part2; // partial sums of the depthwise output: 2 arrays of Cexp*NPdw
    size_t part_floats;
    size_t o_G, o_dy1, o_coef3, o_coef2, o_coef1, o_dg, o_A1, o_A2, o_dt, o_dq, o_dzs, o_pdw, o_wg;
    size_t o_splitk; // partial tiles of a split 1x1 convolution
    size_t scratch_bytes;
    int NT1, NT5; // q-tiles of the expansion / projection conv
    int NPdw;     // partial results per channel of the depthwise kernels
};

mbconv_status check_desc(const mbconv_desc *d)
{
    if (!d)
        return MBCONV_EINVAL;
    if (d->N < 1 || d->Cin < 1 || d->H < 1 || d->W < 1 || d->Cexp < 1 || d->Cout < 1)
        return MBCONV_EINVAL;
    if (d->no_se != 0 && d->no_se != 1)
        return MBCONV_EINVAL;
    if (!d->no_se && d->Cse < 1)
        return MBCONV_EINVAL;
    if (d->activation != MBCONV_ACT_SWISH && d->activation != MBCONV_ACT_RELU6)
        return MBCONV_EINVAL;
    if (d->dtype != MBCONV_F32 && d->dtype != MBCONV_BF16)
        return MBCONV_EINVAL;
    if (d->policy != MBCONV_RECOMPUTE && d->policy != MBCONV_STORE)
        return MBCONV_EINVAL;
    if (!d->has_expand && d->Cexp != d->Cin)
        return MBCONV_EINVAL;
    if (d->residual && (d->stride != 1 || d->Cin != d->Cout))
        return MBCONV_EINVAL;
    if (!(d->bn_eps >= 0.f) || !(d->bn_momentum >= 0.f && d->bn_momentum <= 1.f))
        return MBCONV_EINVAL;
    if (d->k != 3 && d->k != 5)
        return MBCONV_EUNSUPPORTED;
    if (d->stride != 1 && d->stride != 2)
        return MBCONV_EUNSUPPORTED;
    if (d->pad != (d->k - 1) / 2)
        return MBCONV_EUNSUPPORTED;
    if (d->H > 128 || d->W > 128) // a whole plane (with border) must fit in LDS
        return MBCONV_EUNSUPPORTED;
    if ((long long)d->N * d->H * d->W >= (1ll << 31) ||
        (long long)d->N * std::max(d->Cexp, std::max(d->Cin, d->Cout)) >= (1ll << 31))
        return MBCONV_EUNSUPPORTED;
    return MBCONV_OK;
}

// The four 1x1 convolutions of a block as launch_conv1x1 sees them: expansion conv, projection
// conv, projection data gradient, expansion data gradient (training mode; the evaluation-mode
// projection conv with BN3 folded into its epilogue reads the same image).
struct ConvRole {
    bool present, stores;
    int M, K, HW, pro, epi;
};
ConvRole conv_role(const Plan &P, int i)
{
    switch (i) {
    case 0:
        return {P.expand, false, P.Cexp, P.Cin, P.HW, PRO_NONE, EPI_STATS};
    case 1:
        return {true, P.store, P.Cout, P.Cexp, P.HWo, PRO_BNSWISH_GATE, EPI_STATS};
    case 2:
        return {true, false, P.Cexp, P.Cout, P.HWo, PRO_BNBWD, EPI_NONE};
    default:
        return {P.expand, false, P.Cin, P.Cexp, P.HW, PRO_BNBWD, P.res ? EPI_RES : EPI_NONE};
    }
}

Plan make_plan(const mbconv_desc *d)
{
    Plan P = {};
    P.N = d->N;
    P.Cin = d->Cin;
    P.H = d->H;
    P.W = d->W;
    P.Cexp = d->Cexp;
    P.Cse = d->no_se ? 1 : d->Cse;
    P.se = !d->no_se;
    P.Cout = d->Cout;
    P.k = d->k;
    P.s = d->stride;
    P.p = d->pad;
    P.Ho = (d->H + 2 * d->pad - d->k) / d->stride + 1;
    P.Wo = (d->W + 2 * d->pad - d->k) / d->stride + 1;
    P.expand = d->has_expand != 0;
    P.res = d->residual != 0;
    P.bf16 = d->dtype == MBCONV_BF16;
    P.store = d->policy == MBCONV_STORE;
    P.esz = P.bf16 ? 2 : 4;
    P.HW = P.H * P.W;
    P.HWo = P.Ho * P.Wo;
    P.nX = (size_t)P.N * P.Cin * P.HW;
    P.nE = (size_t)P.N * P.Cexp * P.HW;
    P.nD = (size_t)P.N * P.Cexp * P.HWo;
    P.nP = (size_t)P.N * P.Cout * P.HWo;
    {
        const DwShape ds = {P.N, P.Cexp, P.H, P.W, P.Ho, P.Wo, P.k, P.s, P.p};
        P.NPdw = dw_num_partials(ds, P.store && P.expand);
    }
    P.NT1 = conv1x1_num_partials(P.bf16, P.N, P.Cexp, P.Cin, P.HW, false, PRO_NONE, EPI_STATS);
    P.NT5 = conv1x1_num_partials(P.bf16, P.N, P.Cout, P.Cexp, P.HWo, d->policy == MBCONV_STORE,
                                 PRO_BNSWISH_GATE, EPI_STATS);

    size_t o = 0;
    auto take = [&o](size_t bytes) {
        size_t at = o;
        o = align_up(o + bytes);
        return at;
    };
    const size_t f = sizeof(float);
    P.o_e = P.expand ? take(P.nE * P.esz) : kAbsent;
    P.o_d = take(P.nD * P.esz);
    P.o_p = take(P.nP * P.esz);
    P.o_bn1 = P.expand ? take(4 * P.Cexp * f) : kAbsent;
    P.o_bn2 = take(4 * P.Cexp * f);
    P.o_bn3 = take(4 * P.Cout * f);
    P.o_z = take((size_t)P.N * P.Cexp * f);
    P.o_g = take((size_t)P.N * P.Cexp * f);
    P.o_q = take((size_t)P.N * P.Cse * f);
    P.o_s3 = take((size_t)P.N * P.Cexp * f);
    P.o_s4 = take((size_t)P.N * P.Cexp * f);
    P.o_a1 = (P.store && P.expand) ? take(P.nE * P.esz) : kAbsent;
    P.o_sc = P.store ? take(P.nD * P.esz) : kAbsent;
    {
        const ConvRole ro[4] = {conv_role(P, 0), conv_role(P, 1), conv_role(P, 2), conv_role(P, 3)};
        for (int i = 0; i < 4; ++i) {
            const bool use = ro[i].present && conv1x1_uses_weight_image(P.bf16, P.N, ro[i].M, ro[i].K, ro[i].HW,
                                                                          ro[i].stores, ro[i].pro, ro[i].epi);
            P.o_wimg[i] = use ? take(x3_weight_image_bytes(ro[i].M, ro[i].K)) : kAbsent;
            P.wimg_lane_order[i] = use ? conv1x1_image_lane_order(P.bf16, P.N, ro[i].M, ro[i].K, ro[i].HW,
                                                                  ro[i].stores, ro[i].pro, ro[i].epi)
                                       : 0;
        }
    }
    P.saved_bytes = o;

    o = 0;
    size_t part = (size_t)P.Cexp * P.N;                       // depthwise planes
    part = std::max(part, (size_t)P.Cout * P.N);              // BN3 backward planes
    part = std::max(part, (size_t)P.Cout * P.NT5);            // projection conv tiles
    if (P.expand)
        part = std::max(part, (size_t)P.Cexp * P.NT1);        // expansion conv tiles
    P.part_floats = part;
    P.o_part = take(2 * part * f);
    // the depthwise output's partial statistics live apart from the expansion conv's, which the
    // depthwise kernel may still be reading (it finalises BN1 itself)
    P.o_part2 = take(2 * (size_t)P.Cexp * P.NPdw * f);
    P.o_G = take(P.nD * P.esz);
    P.o_dy1 = P.expand ? take(P.nE * P.esz) : kAbsent;
    P.o_coef3 = take(3 * P.Cout * f);
    P.o_coef2 = take(3 * P.Cexp * f);
    P.o_coef1 = P.expand ? take(3 * P.Cexp * f) : kAbsent;
    P.o_dg = take((size_t)P.N * P.Cexp * f);
    P.o_A1 = take((size_t)P.N * P.Cexp * f);
    P.o_A2 = take((size_t)P.N * P.Cexp * f);
    P.o_dt = take((size_t)P.N * P.Cexp * f);
    P.o_dq = take((size_t)P.N * P.Cse * f);
    P.o_dzs = take((size_t)P.N * P.Cexp * f);
    P.o_pdw = take((size_t)P.N * P.Cexp * P.k * P.k * f);
    size_t wg = (size_t)wgrad_splits(P.bf16, P.Cout, P.Cexp, P.N, P.HWo) * P.Cout * P.Cexp;
    if (P.expand)
        wg = std::max(wg, (size_t)wgrad_splits(P.bf16, P.Cexp, P.Cin, P.N, P.HW) * P.Cexp * P.Cin);
    P.o_wg = take(wg * f);
    size_t sk = conv1x1_splitk_floats(P.bf16, P.N, P.Cout, P.Cexp, P.HWo, P.store);
    sk = std::max(sk, conv1x1_splitk_floats(P.bf16, P.N, P.Cexp, P.Cout, P.HWo, false));
    if (P.expand) {
        sk = std::max(sk, conv1x1_splitk_floats(P.bf16, P.N, P.Cexp, P.Cin, P.HW, false));
        sk = std::max(sk, conv1x1_splitk_floats(P.bf16, P.N, P.Cin, P.Cexp, P.HW, false));
    }
    P.o_splitk = take(sk * f);
    P.o_wg2 = P.expand ? take((size_t)wgrad_splits(P.bf16, P.Cout, P.Cexp, P.N, P.HWo) * P.Cout * P.Cexp * f)
                       : kAbsent;
    P.scratch_bytes = o;
    return P;
}

bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

template <typename T>
T *at(void *base, size_t off)
{
    return reinterpret_cast<T *>(static_cast<char *>(base) + off);
}
template <typename T>
const T *at(const void *base, size_t off)
{
    return reinterpret_cast<const T *>(static_cast<const char *>(base) + off);
}

#define MBK_TRY(expr)                                                                             \
    do {                                                                                          \
        if ((expr) != hipSuccess)                                                                 \
            return MBCONV_EHIP;                                                                   \
    } while (0)

// Runs one step of the launch sequence, bracketed by the probe's events when it names it.
#define MBK_STEP(id, expr)                                                                        \
    do {                                                                                          \
        const bool probed_ = probe && probe->step == (id) && probe->start_event &&                \
                             probe->stop_event;                                                   \
        if (probed_)                                                                              \
            MBK_TRY(hipEventRecord((hipEvent_t)probe->start_event, st));                          \
        MBK_TRY(expr);                                                                            \
        if (probed_)                                                                              \
            MBK_TRY(hipEventRecord((hipEvent_t)probe->stop_event, st));                           \
    } while (0)

mbconv_status check_params(const mbconv_desc *d, const mbconv_params *p)
{
    if (!p)
        return MBCONV_EINVAL;
    const void *req[] = {p->w_dw, p->bn2_gamma, p->bn2_beta, p->w_proj, p->bn3_gamma, p->bn3_beta};
    for (const void *q : req)
        if (!q)
            return MBCONV_EINVAL;
    if (!d->no_se && (!p->se_w1 || !p->se_b1 || !p->se_w2 || !p->se_b2))
        return MBCONV_EINVAL;
    if (d->has_expand && (!p->w_expand || !p->bn1_gamma || !p->bn1_beta))
        return MBCONV_EINVAL;
    const void *all[] = {p->w_expand, p->bn1_gamma, p->bn1_beta, p->w_dw,  p->bn2_gamma,
                         p->bn2_beta, p->se_w1,     p->se_b1,    p->se_w2, p->se_b2,
                         p->w_proj,   p->bn3_gamma, p->bn3_beta};
    for (const void *q : all)
        if (q && misaligned(q))
            return MBCONV_EALIGN;
    return MBCONV_OK;
}



} // namespace


// Training mode (eval == false): batch statistics, running statistics updated when run != NULL.
// Evaluation mode: run is read only and supplies the statistics of all three normalisations;
// their coefficient blocks come from one launch ahead of everything else, attributed to the
// first BN-finalise step the block has, and the other finalise steps launch nothing.
mbconv_status forward_impl(const mbconv_desc *desc, const mbconv_params *prm, mbconv_bn_state *run,
                           bool eval, const void *x, void *out, void *saved, void *scratch,
                           void *hip_stream, const mbconv_probe *probe)
{
    mbconv_status s = check_desc(desc);
    if (s != MBCONV_OK)
        return s;
    s = check_params(desc, prm);
    if (s != MBCONV_OK)
        return s;
    if (!x || !out || !saved || !scratch)
        return MBCONV_EINVAL;
    if (misaligned(x) || misaligned(out) || misaligned(saved) || misaligned(scratch))
        return MBCONV_EALIGN;
    if (eval && !run)
        return MBCONV_EINVAL;
    if (run) {
        if (!run->bn2_mean || !run->bn2_var || !run->bn3_mean || !run->bn3_var)
            return MBCONV_EINVAL;
        if (desc->has_expand && (!run->bn1_mean || !run->bn1_var))
            return MBCONV_EINVAL;
        const void *all[] = {run->bn1_mean, run->bn1_var, run->bn2_mean,
                             run->bn2_var,  run->bn3_mean, run->bn3_var};
        for (const void *q : all)
            if (q && ((uintptr_t)q & 3u))
                return MBCONV_EALIGN;
    }
    const Plan P = make_plan(desc);
    hipStream_t st = (hipStream_t)hip_stream;
    const bool bf = P.bf16;
    float *psum = at<float>(scratch, P.o_part);
    float *psq = psum + P.part_floats;
    float *psum2 = at<float>(scratch, P.o_part2);
    float *psq2 = psum2 + (size_t)P.Cexp * P.NPdw;
    float *splitk = at<float>(scratch, P.o_splitk);
    float *bn2 = at<float>(saved, P.o_bn2), *bn3 = at<float>(saved, P.o_bn3);
    float *bn1 = P.expand ? at<float>(saved, P.o_bn1) : nullptr;
    void *d = at<char>(saved, P.o_d), *p = at<char>(saved, P.o_p);
    const float eps = desc->bn_eps, mom = desc->bn_momentum;

    const auto eval_coefs = [&]() {
        return launch_bn_eval_coef(P.expand ? P.Cexp : 0, prm->bn1_gamma, prm->bn1_beta, run->bn1_mean,
                                   run->bn1_var, bn1, P.Cexp, prm->bn2_gamma, prm->bn2_beta,
                                   run->bn2_mean, run->bn2_var, bn2, P.Cout, prm->bn3_gamma,
                                   prm->bn3_beta, run->bn3_mean, run->bn3_var, bn3, eps, st);
    };
    if (eval)
        MBK_STEP(P.expand ? MBCONV_STEP_BN1_FINALIZE : MBCONV_STEP_BN2_FINALIZE, eval_coefs());
    // Weight images of the convolutions that want them (one launch; the two data-gradient images
    // only in training mode).  The launch belongs to the step of the first convolution.
    const auto wimg = [&](int i) -> const void * {
        return P.o_wimg[i] == kAbsent ? nullptr : at<char>(saved, P.o_wimg[i]);
    };
    const auto prep_images = [&]() -> hipError_t {
        const float *w[4];
        int M[4], K[4], sm[4], sk[4], lo[4], n = 0;
        void *img[4];
        const float *we = (const float *)prm->w_expand, *wp = (const float *)prm->w_proj;
        const auto add = [&](int i, const float *src, int m, int k, int s_m, int s_k) {
            if (P.o_wimg[i] == kAbsent)
                return;
            w[n] = src;
            M[n] = m;
            K[n] = k;
            sm[n] = s_m;
            sk[n] = s_k;
            img[n] = at<char>(saved, P.o_wimg[i]);
            lo[n] = P.wimg_lane_order[i];
            ++n;
        };
        add(0, we, P.Cexp, P.Cin, P.Cin, 1);
        add(1, wp, P.Cout, P.Cexp, P.Cexp, 1);
        if (!eval) {
            add(2, wp, P.Cexp, P.Cout, 1, P.Cexp);
            add(3, we, P.Cin, P.Cexp, 1, P.Cin);
        }
        return n ? launch_x3_prep(n, w, M, K, sm, sk, img, lo, st) : hipSuccess;
    };
    bool images_ready = false;
    // expansion conv + BN1 statistics
    const void *dw_in = x;
    if (P.expand) {
        void *e = at<char>(saved, P.o_e);
        Operand B;
        B.p0 = x;
        B.pro = PRO_NONE;
        const auto conv = [&]() -> hipError_t {
            const hipError_t pe = prep_images();
            if (pe != hipSuccess)
                return pe;
            return launch_conv1x1(bf, P.N, P.Cexp, P.Cin, P.HW, prm->w_expand, P.Cin, 1, B, e, EPI_STATS,
                                  nullptr, psum, psq, nullptr, splitk, st, wimg(0));
        };
        MBK_STEP(MBCONV_STEP_EXPAND_CONV, conv());
        images_ready = true;
        dw_in = e;
    }
    // A normalisation's finalise step (partial sums -> scale, shift, mean, rstd, running
    // statistics) runs inside the kernel that first consumes the statistics where that pays (BN1
    // in the vectorised depthwise kernel, BN3 in the final elementwise pass, both for large
    // planes; measured for BN2 in the pooling kernel: no gain); otherwise it is a launch of its own.
    const DwShape ds = {P.N, P.Cexp, P.H, P.W, P.Ho, P.Wo, P.k, P.s, P.p};
    void *a1_store = (P.store && P.expand && !eval) ? at<char>(saved, P.o_a1) : nullptr;
    const double m1 = (double)P.N * P.HW, m2 = (double)P.N * P.HWo;
    const BnFin fin1 = make_bn_fin(psum, psq, prm->bn1_gamma, prm->bn1_beta, run ? run->bn1_mean : nullptr,
                                   run ? run->bn1_var : nullptr, bn1, P.NT1, eps, mom, m1);
    const BnFin fin3 = make_bn_fin(psum, psq, prm->bn3_gamma, prm->bn3_beta, run ? run->bn3_mean : nullptr,
                                   run ? run->bn3_var : nullptr, bn3, P.NT5, eps, mom, m2);
    const bool fuse1 = !eval && P.expand && dw_fwd_finalizes_bn1(ds, a1_store != nullptr);
    const bool fuse3 = !eval && plane_finalize_pays(P.HWo);
    if (P.expand && !eval && !fuse1)
        MBK_STEP(MBCONV_STEP_BN1_FINALIZE, launch_bn_finalize(P.Cexp, P.NT1, m1, psum, psq, prm->bn1_gamma,
                                   prm->bn1_beta, eps, mom, fin1.run_mean, fin1.run_var, bn1, st));
    // BN1 + Swish + depthwise + BN2 statistics
    MBK_STEP(MBCONV_STEP_DW_FWD, launch_dw_fwd(bf, ds, dw_in, bn1, prm->w_dw, d, psum2, psq2, a1_store,
                                               fuse1 ? &fin1 : nullptr, st));
    // BN2 + Swish + SE squeeze, SE excite
    float *z = at<float>(saved, P.o_z), *g = at<float>(saved, P.o_g), *q = at<float>(saved, P.o_q);
    // no squeeze-and-excitation stage: the gate every later prologue multiplies by is one; in
    // training BN2's finalisation writes it
    if (!eval)
        MBK_STEP(MBCONV_STEP_BN2_FINALIZE, launch_bn_finalize(P.Cexp, P.NPdw, m2, psum2, psq2, prm->bn2_gamma,
                                   prm->bn2_beta, eps, mom, run ? run->bn2_mean : nullptr,
                                   run ? run->bn2_var : nullptr, bn2, st, P.se ? nullptr : g,
                                   (size_t)P.N * P.Cexp));
    if (P.se) {
        MBK_STEP(MBCONV_STEP_SE_POOL, launch_pool(bf, P.N, P.Cexp, P.HWo, d, bn2, z, at<float>(saved, P.o_s3),
                            at<float>(saved, P.o_s4), st));
        MBK_STEP(MBCONV_STEP_SE_FC, launch_se_fwd(P.N, P.Cexp, P.Cse, z, prm->se_w1, prm->se_b1, prm->se_w2, prm->se_b2, q,
                              g, st));
    } else if (eval) {
        MBK_STEP(MBCONV_STEP_SE_FC, launch_fill(g, 1.0f, (size_t)P.N * P.Cexp, st));
    }
    // projection conv on Swish(BN2(d))*g + BN3 statistics
    {
        Operand B;
        B.p0 = d;
        B.c0 = bn2;
        B.c1 = bn2 + P.Cexp;
        B.gate = g;
        B.pro = PRO_BNSWISH_GATE;
        if (eval) {
            // BN3 with fixed statistics is an affine map per output channel: it and the residual
            // go into the convolution's epilogue where the kernel family has one
            hipError_t fused = hipSuccess;
            const auto try_fused = [&]() {
                if (!images_ready) { // a block without expansion conv
                    const hipError_t pe = prep_images();
                    if (pe != hipSuccess)
                        return pe;
                    images_ready = true;
                }
                fused = launch_conv1x1_affine(bf, P.N, P.Cout, P.Cexp, P.HWo, prm->w_proj, P.Cexp, 1, B,
                                              out, P.res ? x : nullptr, bn3, bn3 + P.Cout, st, wimg(1));
                return fused == hipErrorNotSupported ? hipSuccess : fused;
            };
            MBK_STEP(MBCONV_STEP_PROJ_CONV, try_fused());
            if (fused == hipSuccess)
                return MBCONV_OK;
        }
        void *sc_store = (P.store && !eval) ? at<char>(saved, P.o_sc) : nullptr;
        const auto conv = [&]() -> hipError_t {
            if (!images_ready) { // a block without expansion conv
                const hipError_t pe = prep_images();
                if (pe != hipSuccess)
                    return pe;
                images_ready = true;
            }
            return launch_conv1x1(bf, P.N, P.Cout, P.Cexp, P.HWo, prm->w_proj, P.Cexp, 1, B, p, EPI_STATS,
                                  nullptr, psum, psq, sc_store, splitk, st, wimg(1));
        };
        MBK_STEP(MBCONV_STEP_PROJ_CONV, conv());
        if (!eval && !fuse3)
            MBK_STEP(MBCONV_STEP_BN3_FINALIZE, launch_bn_finalize(P.Cout, P.NT5, m2, psum, psq, prm->bn3_gamma,
                                       prm->bn3_beta, eps, mom, fin3.run_mean, fin3.run_var, bn3, st));
    }
    // BN3 (+ residual), finalising BN3's statistics on the way in training mode
    MBK_STEP(MBCONV_STEP_BN3_APPLY, launch_bn_apply(bf, P.N, P.Cout, P.HWo, p, bn3, P.res ? x : nullptr, out,
                                                    fuse3 ? &fin3 : nullptr, st));
    return MBCONV_OK;
}


mbconv_status backward_impl(const mbconv_desc *desc, const mbconv_params *prm, const void *x,
                            const void *dout, const void *saved, void *scratch, void *dx,
                            mbconv_grads *gr, void *hip_stream, const mbconv_probe *probe)
{
    mbconv_status s = check_desc(desc);
    if (s != MBCONV_OK)
        return s;
    s = check_params(desc, prm);
    if (s != MBCONV_OK)
        return s;
    if (!x || !dout || !saved || !scratch || !dx || !gr)
        return MBCONV_EINVAL;
    if (misaligned(x) || misaligned(dout) || misaligned(saved) || misaligned(scratch) ||
        misaligned(dx))
        return MBCONV_EALIGN;
    {
        const void *req[] = {gr->w_dw, gr->bn2_gamma, gr->bn2_beta, gr->w_proj, gr->bn3_gamma, gr->bn3_beta};
        for (const void *q : req)
            if (!q)
                return MBCONV_EINVAL;
        if (!desc->no_se && (!gr->se_w1 || !gr->se_b1 || !gr->se_w2 || !gr->se_b2))
            return MBCONV_EINVAL;
        if (desc->has_expand && (!gr->w_expand || !gr->bn1_gamma || !gr->bn1_beta))
            return MBCONV_EINVAL;
    }
    const Plan P = make_plan(desc);
    hipStream_t st = (hipStream_t)hip_stream;
    const bool bf = P.bf16;
    float *pa = at<float>(scratch, P.o_part);
    float *pb = pa + P.part_floats;
    const float *bn2 = at<float>(saved, P.o_bn2), *bn3 = at<float>(saved, P.o_bn3);
    const float *bn1 = P.expand ? at<float>(saved, P.o_bn1) : nullptr;
    const void *d = at<char>(saved, P.o_d), *p = at<char>(saved, P.o_p);
    const float *z = at<float>(saved, P.o_z), *g = at<float>(saved, P.o_g);
    const float *q = at<float>(saved, P.o_q);
    float *coef3 = at<float>(scratch, P.o_coef3), *coef2 = at<float>(scratch, P.o_coef2);
    void *G = at<char>(scratch, P.o_G);
    float *wg = at<float>(scratch, P.o_wg), *splitk = at<float>(scratch, P.o_splitk);
    const double m2 = (double)P.N * P.HWo;

    // BN3 backward reductions
    MBK_STEP(MBCONV_STEP_BN3_BWD_REDUCE, launch_plane_dot(bf, P.N, P.Cout, P.HWo, dout, p, bn3, pa, pb, st));
    // (where one kernel computes both gradients of the projection conv, it also finalises BN3's
    // backward: no launch for that step)
    int psplits = 0;
    const bool proj_fused = projbwd_fused_plan(P.N, P.Cexp, P.Cout, P.HWo, &psplits);
    const BnBwdFin fin3 = {pa, pb, prm->bn3_gamma, bn3, gr->bn3_gamma, gr->bn3_beta, coef3, P.N, m2};
    if (!proj_fused)
        MBK_STEP(MBCONV_STEP_BN3_BWD_FINALIZE, launch_bn_bwd_finalize(P.Cout, P.N, m2, pa, pb, prm->bn3_gamma, bn3,
                                       gr->bn3_gamma, gr->bn3_beta, coef3, st));
    // projection conv: data gradient G = W_p^T dp and weight gradient dW_p = dp * sc^T,
    // dp rebuilt in the prologue from dout and p
    SplitReduce proj_reduce = {nullptr, 0, 0, nullptr};
    bool pair_wgrads = false; // the projection conv's weight gradient shares the expansion conv's launch
    Operand pair_dp, pair_sc;
    float *pair_pwg = nullptr;
    Operand dp;
    dp.p0 = dout;
    dp.p1 = p;
    dp.c0 = coef3;
    dp.c1 = coef3 + P.Cout;
    dp.c2 = coef3 + 2 * P.Cout;
    dp.pro = PRO_BNBWD;
    {
        Operand sc;
        if (P.store) {
            sc.p0 = at<char>(saved, P.o_sc);
            sc.pro = PRO_NONE;
        } else {
            sc.p0 = d;
            sc.c0 = bn2;
            sc.c1 = bn2 + P.Cexp;
            sc.gate = g;
            sc.pro = PRO_BNSWISH_GATE;
        }
        // with an expansion conv, the sum over this weight gradient's splits waits for the
        // other's and shares its launch (the partials then live in a region of their own)
        float *pwg = P.expand ? at<float>(scratch, P.o_wg2) : wg;
        if (proj_fused) {
            // one kernel for both gradients (its launch is the PROJ_DGRAD step)
            MBK_STEP(MBCONV_STEP_PROJ_DGRAD, launch_projbwd_fused(bf, P.N, P.Cexp, P.Cout, P.HWo, dp, sc, prm->w_proj,
                                                                  G, pwg, &psplits, &fin3, st));
            proj_reduce = {pwg, psplits, (size_t)P.Cout * P.Cexp, gr->w_proj};
            if (!P.expand)
                MBK_STEP(MBCONV_STEP_PROJ_WGRAD,
                         launch_reduce_splits2(proj_reduce, {nullptr, 0, 0, nullptr}, st));
        } else {
            MBK_STEP(MBCONV_STEP_PROJ_DGRAD, launch_conv1x1(bf, P.N, P.Cexp, P.Cout, P.HWo, prm->w_proj, 1, P.Cexp, dp,
                                                            G, EPI_NONE, nullptr, nullptr, nullptr, nullptr, splitk, st,
                                                            P.o_wimg[2] == kAbsent ? nullptr : at<char>(saved, P.o_wimg[2])));
            // where both weight gradients of the block are shapes of the split-operand kernel and
            // the expansion conv's backward is not a fused kernel, this one waits and shares the
            // other's launch (its operands stay as they are until the end of the pass)
            int fs = 0;
            pair_wgrads = P.expand && !bwd1x1_fused_plan(P.N, P.Cexp, P.Cin, P.HW, &fs) &&
                          wgrad1x1_pair_supported(bf, P.N, P.Cout, P.Cexp, P.HWo, P.Cexp, P.Cin, P.HW);
            if (pair_wgrads) {
                pair_dp = dp;
                pair_sc = sc;
                pair_pwg = pwg;
            } else {
                MBK_STEP(MBCONV_STEP_PROJ_WGRAD,
                         launch_wgrad1x1(bf, P.N, P.Cout, P.Cexp, P.HWo, dp, sc, pwg, gr->w_proj,
                                         P.expand ? &proj_reduce : nullptr, st));
            }
        }
    }
    // SE backward and BN2 backward reductions
    float *dg = at<float>(scratch, P.o_dg), *A1 = at<float>(scratch, P.o_A1);
    float *A2 = at<float>(scratch, P.o_A2), *dzs = at<float>(scratch, P.o_dzs);
    MBK_STEP(MBCONV_STEP_GATE_SUMS, launch_gate_sums(bf, P.N, P.Cexp, P.HWo, G, d, bn2, dg, A1, A2, st));
    if (!P.se) {
        // gate = 1, dz = 0: BN2's parameter gradients are the batch sums of the plane sums
        MBK_STEP(MBCONV_STEP_SE_BWD, launch_bn2_bwd_nose(P.N, P.Cexp, (double)P.N * P.HWo, A1, A2, prm->bn2_gamma, bn2,
                                                         gr->bn2_gamma, gr->bn2_beta, coef2, dzs, st));
    } else {
        SeBwdArgs a;
        a.N = P.N;
        a.C = P.Cexp;
        a.Cse = P.Cse;
        a.HW = P.HWo;
        a.z = z;
        a.g = g;
        a.q = q;
        a.w1 = prm->se_w1;
        a.w2 = prm->se_w2;
        a.dg = dg;
        a.A1 = A1;
        a.A2 = A2;
        a.s3 = at<float>(saved, P.o_s3);
        a.s4 = at<float>(saved, P.o_s4);
        a.gamma2 = prm->bn2_gamma;
        a.bn2 = bn2;
        a.dt = at<float>(scratch, P.o_dt);
        a.dq = at<float>(scratch, P.o_dq);
        a.dzs = dzs;
        a.dw1 = gr->se_w1;
        a.db1 = gr->se_b1;
        a.dw2 = gr->se_w2;
        a.db2 = gr->se_b2;
        a.dgamma2 = gr->bn2_gamma;
        a.dbeta2 = gr->bn2_beta;
        a.coef2 = coef2;
        MBK_STEP(MBCONV_STEP_SE_BWD, launch_se_bwd(a, st));
    }
    // fused depthwise backward
    {
        DwBwdArgs a;
        a.s = {P.N, P.Cexp, P.H, P.W, P.Ho, P.Wo, P.k, P.s, P.p};
        a.G = G;
        a.d = d;
        a.e = P.expand ? at<char>(saved, P.o_e) : x;
        a.g = g;
        a.dzs = dzs;
        a.bn2 = bn2;
        a.coef2 = coef2;
        a.bn1 = bn1;
        a.w_dw = prm->w_dw;
        a.a1_saved = (P.store && P.expand) ? at<char>(saved, P.o_a1) : nullptr;
        a.dy1_out = P.expand ? at<char>(scratch, P.o_dy1) : dx;
        a.res = (!P.expand && P.res) ? dout : nullptr;
        a.pdw = at<float>(scratch, P.o_pdw);
        a.psb = pa;
        a.psr = pb;
        MBK_STEP(MBCONV_STEP_DW_BWD, launch_dw_bwd(bf, a, st));
        if (P.expand) {
            // one launch: filter-gradient partials and BN1's backward finalisation
            MBK_STEP(MBCONV_STEP_DW_WGRAD_REDUCE,
                     launch_dw_bwd_finalize(a.pdw, P.Cexp, P.NPdw, P.k * P.k, gr->w_dw, (double)P.N * P.HW, pa,
                                            pb, prm->bn1_gamma, bn1, gr->bn1_gamma, gr->bn1_beta,
                                            at<float>(scratch, P.o_coef1), st));
        } else {
            MBK_STEP(MBCONV_STEP_DW_WGRAD_REDUCE, launch_reduce_planes(a.pdw, P.Cexp, P.NPdw, P.k * P.k, gr->w_dw, st));
        }
    }
    if (P.expand) {
        float *coef1 = at<float>(scratch, P.o_coef1);
        const void *e = at<char>(saved, P.o_e);
        const void *dy1 = at<char>(scratch, P.o_dy1);
        MBK_STEP(MBCONV_STEP_BN1_BWD_FINALIZE, hipSuccess); // done by the launch above
        Operand de;
        de.p0 = dy1;
        de.p1 = e;
        de.c0 = coef1;
        de.c1 = coef1 + P.Cexp;
        de.c2 = coef1 + 2 * P.Cexp;
        de.pro = PRO_BNBWD;
        // dx = W_e^T de (+ dout), dW_e = de * x^T: one pass over de where the fused kernel covers
        // the shape (its launch is the EXPAND_DGRAD step, the sums over the splits EXPAND_WGRAD)
        int fsplits = 0;
        if (bwd1x1_fused_plan(P.N, P.Cexp, P.Cin, P.HW, &fsplits)) {
            MBK_STEP(MBCONV_STEP_EXPAND_DGRAD,
                     launch_bwd1x1_fused(bf, P.N, P.Cexp, P.Cin, P.HW, de, x, prm->w_expand, dx,
                                         P.res ? dout : nullptr, wg, &fsplits, st));
            const SplitReduce exp_reduce = {wg, fsplits, (size_t)P.Cexp * P.Cin, gr->w_expand};
            MBK_STEP(MBCONV_STEP_EXPAND_WGRAD, launch_reduce_splits2(exp_reduce, proj_reduce, st));
            return MBCONV_OK;
        }
        MBK_STEP(MBCONV_STEP_EXPAND_DGRAD, launch_conv1x1(bf, P.N, P.Cin, P.Cexp, P.HW, prm->w_expand, 1, P.Cin, de, dx,
                               P.res ? EPI_RES : EPI_NONE, P.res ? dout : nullptr, nullptr, nullptr,
                               nullptr, splitk, st,
                               P.o_wimg[3] == kAbsent ? nullptr : at<char>(saved, P.o_wimg[3])));
        Operand xo;
        xo.p0 = x;
        xo.pro = PRO_NONE;
        const auto both = [&]() {
            SplitReduce exp_reduce;
            hipError_t e;
            if (pair_wgrads)
                e = launch_wgrad1x1_pair(bf, P.N, P.Cout, P.Cexp, P.HWo, pair_dp, pair_sc, pair_pwg, gr->w_proj,
                                         &proj_reduce, P.Cexp, P.Cin, P.HW, de, xo, wg, gr->w_expand,
                                         &exp_reduce, st);
            else
                e = launch_wgrad1x1(bf, P.N, P.Cexp, P.Cin, P.HW, de, xo, wg, gr->w_expand, &exp_reduce, st);
            return e != hipSuccess ? e : launch_reduce_splits2(exp_reduce, proj_reduce, st);
        };
        MBK_STEP(MBCONV_STEP_EXPAND_WGRAD, both());
    }
    return MBCONV_OK;
}


} // namespace mbk

#ifndef MBK_ACT_RELU6
using namespace mbk;

namespace mbk_r6 {
mbconv_status forward_impl(const mbconv_desc *desc, const mbconv_params *prm, mbconv_bn_state *run,
                           bool eval, const void *x, void *out, void *saved, void *scratch,
                           void *hip_stream, const mbconv_probe *probe);
mbconv_status backward_impl(const mbconv_desc *desc, const mbconv_params *prm, const void *x,
                            const void *dout, const void *saved, void *scratch, void *dx,
                            mbconv_grads *gr, void *hip_stream, const mbconv_probe *probe);
} // namespace mbk_r6

namespace {
bool relu6(const mbconv_desc *d) { return d && d->activation == MBCONV_ACT_RELU6; }
} // namespace

extern "C" {

int32_t mbconv_abi_version(void) { return 4; }

mbconv_status mbconv_step_engine(const mbconv_desc *desc, int32_t step, int32_t *engine)
{
    const mbconv_status s = check_desc(desc);
    if (s != MBCONV_OK)
        return s;
    if (!engine || step <= MBCONV_STEP_NONE || step >= MBCONV_STEP_COUNT)
        return MBCONV_EINVAL;
    const Plan P = make_plan(desc);
    int e = MBCONV_ENGINE_VECTOR;
    switch (step) {
    case MBCONV_STEP_EXPAND_CONV:
        if (P.expand)
            e = conv1x1_engine(P.bf16, P.N, P.Cexp, P.Cin, P.HW, false, PRO_NONE, EPI_STATS);
        break;
    case MBCONV_STEP_PROJ_CONV:
        e = conv1x1_engine(P.bf16, P.N, P.Cout, P.Cexp, P.HWo, P.store);
        break;
    case MBCONV_STEP_PROJ_DGRAD:
    case MBCONV_STEP_PROJ_WGRAD: {
        int ps = 0;
        const bool fused = projbwd_fused_plan(P.N, P.Cexp, P.Cout, P.HWo, &ps);
        if (step == MBCONV_STEP_PROJ_DGRAD)
            e = fused ? MBCONV_ENGINE_MFMA_F32 : conv1x1_engine(P.bf16, P.N, P.Cexp, P.Cout, P.HWo, false, PRO_BNBWD, EPI_NONE);
        else
            e = fused ? MBCONV_ENGINE_VECTOR : wgrad1x1_engine(P.bf16, P.Cout, P.Cexp, P.N, P.HWo);
        break;
    }
    case MBCONV_STEP_EXPAND_DGRAD:
    case MBCONV_STEP_EXPAND_WGRAD:
        if (P.expand) {
            int fs = 0;
            const bool fused = bwd1x1_fused_plan(P.N, P.Cexp, P.Cin, P.HW, &fs);
            if (step == MBCONV_STEP_EXPAND_DGRAD)
                e = fused ? bwd1x1_fused_engine(P.bf16, P.N, P.Cexp, P.Cin, P.HW)
                          : conv1x1_engine(P.bf16, P.N, P.Cin, P.Cexp, P.HW, false);
            else
                e = fused ? MBCONV_ENGINE_VECTOR : wgrad1x1_engine(P.bf16, P.Cexp, P.Cin, P.N, P.HW);
        }
        break;
    default:
        break;
    }
    *engine = e;
    return MBCONV_OK;
}

const char *mbconv_status_string(mbconv_status s)
{
    switch (s) {
    case MBCONV_OK:
        return "ok";
    case MBCONV_EINVAL:
        return "invalid argument";
    case MBCONV_EUNSUPPORTED:
        return "unsupported shape";
    case MBCONV_EWORKSPACE:
        return "workspace too small";
    case MBCONV_EALIGN:
        return "pointer not 16-byte aligned";
    case MBCONV_EHIP:
        return "HIP launch failed";
    }
    return "unknown status";
}

mbconv_status mbconv_workspace_size(const mbconv_desc *desc, size_t *saved_bytes,
                                    size_t *scratch_bytes)
{
    mbconv_status s = check_desc(desc);
    if (s != MBCONV_OK)
        return s;
    if (!saved_bytes || !scratch_bytes)
        return MBCONV_EINVAL;
    const Plan P = make_plan(desc);
    *saved_bytes = P.saved_bytes;
    *scratch_bytes = P.scratch_bytes;
    return MBCONV_OK;
}

mbconv_status mbconv_saved_offsets(const mbconv_desc *desc, mbconv_saved_layout *L)
{
    mbconv_status s = check_desc(desc);
    if (s != MBCONV_OK)
        return s;
    if (!L)
        return MBCONV_EINVAL;
    const Plan P = make_plan(desc);
    L->e = P.o_e;
    L->d = P.o_d;
    L->p = P.o_p;
    L->bn1 = P.o_bn1;
    L->bn2 = P.o_bn2;
    L->bn3 = P.o_bn3;
    L->z = P.o_z;
    L->g = P.o_g;
    L->q = P.o_q;
    L->a1 = P.o_a1;
    L->sc = P.o_sc;
    return MBCONV_OK;
}

mbconv_status mbconv_forward(const mbconv_desc *desc, const mbconv_params *prm,
                             mbconv_bn_state *run, const void *x, void *out, void *saved,
                             void *scratch, void *hip_stream)
{
    return mbconv_forward_probed(desc, prm, run, x, out, saved, scratch, hip_stream, nullptr);
}

mbconv_status mbconv_forward_probed(const mbconv_desc *desc, const mbconv_params *prm,
                                    mbconv_bn_state *run, const void *x, void *out, void *saved,
                                    void *scratch, void *hip_stream, const mbconv_probe *probe)
{
    return relu6(desc) ? mbk_r6::forward_impl(desc, prm, run, false, x, out, saved, scratch, hip_stream, probe)
                       : mbk::forward_impl(desc, prm, run, false, x, out, saved, scratch, hip_stream, probe);
}

mbconv_status mbconv_eval_workspace_size(const mbconv_desc *desc, size_t *workspace_bytes)
{
    mbconv_status s = check_desc(desc);
    if (s != MBCONV_OK)
        return s;
    if (!workspace_bytes)
        return MBCONV_EINVAL;
    const Plan P = make_plan(desc);
    *workspace_bytes = align_up(P.saved_bytes) + P.scratch_bytes;
    return MBCONV_OK;
}

mbconv_status mbconv_forward_eval(const mbconv_desc *desc, const mbconv_params *prm,
                                  const mbconv_bn_state *running, const void *x, void *out,
                                  void *workspace, void *hip_stream)
{
    return mbconv_forward_eval_probed(desc, prm, running, x, out, workspace, hip_stream, nullptr);
}

mbconv_status mbconv_forward_eval_probed(const mbconv_desc *desc, const mbconv_params *prm,
                                         const mbconv_bn_state *running, const void *x, void *out,
                                         void *workspace, void *hip_stream,
                                         const mbconv_probe *probe)
{
    mbconv_status s = check_desc(desc);
    if (s != MBCONV_OK)
        return s;
    if (!running || !workspace)
        return MBCONV_EINVAL;
    if (misaligned(workspace))
        return MBCONV_EALIGN;
    const Plan P = make_plan(desc);
    // the intermediates a training call would save, then its scratch region
    char *saved = static_cast<char *>(workspace);
    char *scratch = saved + align_up(P.saved_bytes);
    mbconv_bn_state *run = const_cast<mbconv_bn_state *>(running); // read only in evaluation mode
    return relu6(desc) ? mbk_r6::forward_impl(desc, prm, run, true, x, out, saved, scratch, hip_stream, probe)
                       : mbk::forward_impl(desc, prm, run, true, x, out, saved, scratch, hip_stream, probe);
}

mbconv_status mbconv_backward(const mbconv_desc *desc, const mbconv_params *prm, const void *x,
                              const void *dout, const void *saved, void *scratch, void *dx,
                              mbconv_grads *gr, void *hip_stream)
{
    return mbconv_backward_probed(desc, prm, x, dout, saved, scratch, dx, gr, hip_stream, nullptr);
}

mbconv_status mbconv_backward_probed(const mbconv_desc *desc, const mbconv_params *prm,
                                     const void *x, const void *dout, const void *saved,
                                     void *scratch, void *dx, mbconv_grads *gr, void *hip_stream,
                                     const mbconv_probe *probe)
{
    return relu6(desc) ? mbk_r6::backward_impl(desc, prm, x, dout, saved, scratch, dx, gr, hip_stream, probe)
                       : mbk::backward_impl(desc, prm, x, dout, saved, scratch, dx, gr, hip_stream, probe);
}

} // extern "C"
#endif // MBK_ACT_RELU6
