/*
 * mbconv.h - C ABI of libmbconv: one training step (forward and backward) of an
 * EfficientNet MBConv block on one AMD MI355X (gfx950).
 *
 * The block is the one the paper optimises by hand in its EfficientNet case study
 * (section "Guided Optimization Case Study: EfficientNet"): 1x1 expansion conv ->
 * BN -> Swish -> kxk depthwise conv -> BN -> Swish -> squeeze-and-excitation ->
 * 1x1 projection conv -> BN -> optional residual.  Batch normalisation is the
 * formula of section "Statistical Normalization" taken over (N,H,W) per channel
 * with batch statistics, and it updates running mean/variance as that section
 * says training-mode BN does.  What backward needs is either recomputed from the
 * pre-normalisation tensors or stored, the choice the paper describes in section
 * "Backpropagation and Data Movement".
 *
 * Conventions
 *   - Every tensor is NCHW, contiguous, W fastest.  Ho = (H+2*pad-k)/stride+1.
 *   - "dtype" is the storage type of activation-sized tensors and of the three
 *     convolution weights (fp32, or bf16 with round-to-nearest-even).  BN
 *     parameters and state, SE parameters and every parameter gradient are fp32.
 *     All accumulation is fp32 or wider.
 *   - Every pointer below is a DEVICE pointer unless stated otherwise, owned by the
 *     caller, and must be 16-byte aligned.  The library allocates nothing, keeps no
 *     state between calls and never synchronises: all work is enqueued on the
 *     hipStream_t passed as `hip_stream` (NULL = the default stream).
 *   - Descriptors and the pointer structs themselves live in HOST memory and are
 *     read during the call only.
 *   - Errors: every argument check happens on the host before the first launch and
 *     returns a negative status without touching device memory.  A failed launch
 *     returns MBCONV_EHIP.  Nothing throws, nothing aborts.
 */
#ifndef MBCONV_H
#define MBCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MBCONV_OK = 0,
    MBCONV_EINVAL = -1,       /* null pointer or inconsistent descriptor */
    MBCONV_EUNSUPPORTED = -2, /* shape outside what the kernels cover */
    MBCONV_EWORKSPACE = -3,   /* reserved */
    MBCONV_EALIGN = -4,       /* a pointer is not 16-byte aligned */
    MBCONV_EHIP = -5          /* a HIP launch failed */
} mbconv_status;

typedef enum { MBCONV_F32 = 0, MBCONV_BF16 = 1 } mbconv_dtype;

/* What forward keeps for backward (section "Backpropagation and Data Movement").
 * RECOMPUTE keeps only the three pre-normalisation tensors e, d, p and O(N*C)
 * statistics; backward rebuilds Swish(BN(.)) from them.  STORE additionally keeps the
 * depthwise input a1 = Swish(BN1(e)) and the projection input sc = Swish(BN2(d))*g, and
 * backward reads those instead of rebuilding them. */
typedef enum { MBCONV_RECOMPUTE = 0, MBCONV_STORE = 1 } mbconv_policy;

/* The block's activation after BN1 and after BN2.  Swish is the EfficientNet MBConv block;
 * ReLU6 = min(max(t,0),6) (derivative 1 strictly inside (0,6), else 0) together with no_se = 1
 * is the MobileNet-V2 inverted-residual block, which the paper also times (table "Automatic
 * optimization results").  The SE stage, when present, keeps its own Swish and sigmoid. */
typedef enum { MBCONV_ACT_SWISH = 0, MBCONV_ACT_RELU6 = 1 } mbconv_activation;

typedef struct {
    int32_t N, Cin, H, W; /* input x is [N,Cin,H,W] */
    int32_t Cexp;         /* expanded channels; must equal Cin when has_expand == 0 */
    int32_t Cse, Cout;    /* SE bottleneck width, output channels */
    int32_t k, stride, pad; /* depthwise: k in {3,5}, stride in {1,2}, pad == (k-1)/2 */
    int32_t has_expand;   /* 0: no expansion conv, no BN1, no first Swish (expand ratio 1) */
    int32_t residual;     /* 1: out += x; requires stride == 1 and Cin == Cout */
    int32_t dtype;        /* mbconv_dtype */
    int32_t policy;       /* mbconv_policy */
    float bn_eps;         /* added to the biased batch variance */
    float bn_momentum;    /* running <- (1-momentum)*running + momentum*batch */
    int32_t activation;   /* mbconv_activation */
    int32_t no_se;        /* 1: no squeeze-and-excitation stage (the projection conv consumes the
                             activation of BN2 directly); Cse and the se_* members are ignored */
} mbconv_desc;

/* Parameters, read-only in both calls. */
typedef struct {
    const void *w_expand;               /* [Cexp,Cin]   dtype; NULL iff !has_expand */
    const float *bn1_gamma, *bn1_beta;  /* [Cexp]; NULL iff !has_expand */
    const void *w_dw;                   /* [Cexp,k,k]   dtype */
    const float *bn2_gamma, *bn2_beta;  /* [Cexp] */
    const float *se_w1, *se_b1;         /* [Cse,Cexp], [Cse]; ignored (may be NULL) when no_se */
    const float *se_w2, *se_b2;         /* [Cexp,Cse], [Cexp]; ignored (may be NULL) when no_se */
    const void *w_proj;                 /* [Cout,Cexp]  dtype */
    const float *bn3_gamma, *bn3_beta;  /* [Cout] */
} mbconv_params;

/* Running statistics, updated in place by mbconv_forward.  The variance entering the
 * update is the unbiased batch estimate.  bn1_* may be NULL iff !has_expand. */
typedef struct {
    float *bn1_mean, *bn1_var; /* [Cexp] */
    float *bn2_mean, *bn2_var; /* [Cexp] */
    float *bn3_mean, *bn3_var; /* [Cout] */
} mbconv_bn_state;

/* Parameter gradients, all fp32, same shapes as mbconv_params; OVERWRITTEN, never
 * accumulated.  w_expand, bn1_gamma, bn1_beta may be NULL iff !has_expand; the se_* members
 * are not touched (may be NULL) when no_se. */
typedef struct {
    float *w_expand;
    float *bn1_gamma, *bn1_beta;
    float *w_dw;
    float *bn2_gamma, *bn2_beta;
    float *se_w1, *se_b1;
    float *se_w2, *se_b2;
    float *w_proj;
    float *bn3_gamma, *bn3_beta;
} mbconv_grads;

/* Byte offsets of the named tensors inside the saved workspace, for inspection by
 * tests and tools (SIZE_MAX where a tensor is absent for this descriptor).
 * e, d, p, a1, sc are stored in `dtype`; the rest are fp32.
 * bnX holds four consecutive [C] arrays: scale = gamma*rstd, shift = beta-mean*scale,
 * mean, rstd. */
typedef struct {
    size_t e;   /* [N,Cexp,H,W]   expansion conv output, before BN1 */
    size_t d;   /* [N,Cexp,Ho,Wo] depthwise conv output, before BN2 */
    size_t p;   /* [N,Cout,Ho,Wo] projection conv output, before BN3 */
    size_t bn1, bn2, bn3;
    size_t z;   /* [N,Cexp] SE squeeze (plane means of Swish(BN2(d))) */
    size_t g;   /* [N,Cexp] SE gate */
    size_t q;   /* [N,Cse]  SE hidden pre-activation */
    size_t a1;  /* [N,Cexp,H,W]   STORE policy only */
    size_t sc;  /* [N,Cexp,Ho,Wo] STORE policy only */
} mbconv_saved_layout;

/* Host-only queries.  Both validate the descriptor (MBCONV_EINVAL / MBCONV_EUNSUPPORTED).
 * saved_bytes: what forward writes and the matching backward reads.
 * scratch_bytes: temporary storage either call may overwrite; it can be shared by every
 * block of a network provided it is as large as the largest request. */
mbconv_status mbconv_workspace_size(const mbconv_desc *desc, size_t *saved_bytes,
                                    size_t *scratch_bytes);
mbconv_status mbconv_saved_offsets(const mbconv_desc *desc, mbconv_saved_layout *layout);

/* Forward, training mode.
 *   x   [N,Cin,H,W] dtype, read-only.      out [N,Cout,Ho,Wo] dtype, written.
 *   running: updated in place (may be NULL as a whole to skip the running update).
 *   saved_ws: at least saved_bytes, written; must reach the matching backward unmodified.
 *   scratch_ws: at least scratch_bytes, overwritten. */
mbconv_status mbconv_forward(const mbconv_desc *desc, const mbconv_params *params,
                             mbconv_bn_state *running, const void *x, void *out, void *saved_ws,
                             void *scratch_ws, void *hip_stream);

/* Evaluation-mode forward: every BN normalises with the running statistics instead of the
 * batch's (the paper lists BN among the operators that behave differently in inference and
 * notes that inference stores no activations for backpropagation: section "Background and
 * Related Work", paragraph "Training vs. inference compilation").  Computes
 *   y = gamma*(v - run_mean)/sqrt(run_var + bn_eps) + beta
 * at the three normalisations and otherwise the same block as mbconv_forward.
 *   running: read only, required; bn1_* may be NULL iff !has_expand.
 *   x, out: as for mbconv_forward.   desc->policy is ignored (nothing is saved).
 *   workspace: at least the byte count mbconv_eval_workspace_size reports (host-only query,
 *   same descriptor checks as mbconv_workspace_size); overwritten, nothing in it needs to
 *   survive the call.
 * The _probed variant brackets one step like mbconv_forward_probed; the coefficient blocks of
 * all three normalisations come from one launch attributed to MBCONV_STEP_BN1_FINALIZE
 * (MBCONV_STEP_BN2_FINALIZE when has_expand == 0), the other finalise steps do not occur. */
mbconv_status mbconv_eval_workspace_size(const mbconv_desc *desc, size_t *workspace_bytes);
mbconv_status mbconv_forward_eval(const mbconv_desc *desc, const mbconv_params *params,
                                  const mbconv_bn_state *running, const void *x, void *out,
                                  void *workspace, void *hip_stream);

/* Backward of the forward call that wrote saved_ws (same desc, params and x; the parameter VALUES
 * must be those forward saw as well: for fp32 wide blocks saved_ws holds a re-encoded copy of the
 * two 1x1 conv weights, which the data-gradient kernels read instead of params).
 *   dout [N,Cout,Ho,Wo] dtype, read-only.   dx [N,Cin,H,W] dtype, written.
 *   grads: every non-NULL member is overwritten with the gradient of sum(out*dout).
 * Every reduction runs in a fixed order without floating-point atomics, so results are
 * bitwise repeatable (the paper removes backward atomics by map fission, section
 * "Guided Optimization Case Study: EfficientNet"). */
mbconv_status mbconv_backward(const mbconv_desc *desc, const mbconv_params *params, const void *x,
                              const void *dout, const void *saved_ws, void *scratch_ws, void *dx,
                              mbconv_grads *grads, void *hip_stream);

/* Optional timing probe.  The steps of the two calls, in launch order; a probe brackets
 * exactly one of them with two caller-created HIP events recorded on the call's stream
 * (hipEventRecord(start) before the step's first launch, hipEventRecord(stop) after its last),
 * so a caller can time one kernel inside the timed region without synchronising.
 * The library neither creates, waits on nor destroys the events. */
typedef enum {
    MBCONV_STEP_NONE = 0,
    /* forward */
    MBCONV_STEP_EXPAND_CONV = 1,   /* 1x1 expansion conv + BN1 partial statistics; for fp32 wide blocks also the
                                      launch that re-encodes the 1x1 conv weights (in PROJ_CONV when
                                      has_expand == 0) */
    MBCONV_STEP_BN1_FINALIZE = 2,  /* BN1_FINALIZE and BN3_FINALIZE do not occur where the kernel
                                      that consumes the statistics finalises them itself: DW_FWD
                                      and BN3_APPLY do for planes of 1024 elements or more (DW_FWD:
                                      stride 1, W % 4 == 0, recompute policy) */
    MBCONV_STEP_DW_FWD = 3,        /* BN1 + Swish + depthwise conv + BN2 partial statistics */
    MBCONV_STEP_BN2_FINALIZE = 4,  /* when no_se, in training: also fills the gate with ones */
    MBCONV_STEP_SE_POOL = 5,       /* BN2 + Swish + plane means; does not occur when no_se */
    MBCONV_STEP_SE_FC = 6,         /* when no_se: fills the gate with ones in evaluation mode and does not
                                      occur in training */
    MBCONV_STEP_PROJ_CONV = 7,     /* (BN2 + Swish)*gate + 1x1 projection conv + BN3 partials */
    MBCONV_STEP_BN3_FINALIZE = 8,
    MBCONV_STEP_BN3_APPLY = 9,     /* BN3 (+ residual) */
    /* backward */
    MBCONV_STEP_BN3_BWD_REDUCE = 10,
    MBCONV_STEP_BN3_BWD_FINALIZE = 11, /* does not occur where PROJ_DGRAD is the one-kernel form, which
                                          finalises BN3's backward itself */
    MBCONV_STEP_PROJ_DGRAD = 12,   /* for Cout <= 32 (and H*W a multiple of 4) one kernel computes the
                                      data gradient and the weight gradient's split partial sums */
    MBCONV_STEP_PROJ_WGRAD = 13,   /* with an expansion conv: the split partial sums only, their sum is
                                      part of EXPAND_WGRAD's last launch; does not occur where the two 1x1
                                      weight gradients of the block share one launch (wide blocks whose
                                      two gradients take the same kernel family): that launch is
                                      EXPAND_WGRAD's first */
    MBCONV_STEP_GATE_SUMS = 14,
    MBCONV_STEP_SE_BWD = 15,       /* when no_se: BN2's parameter gradients and backward coefficients only */
    MBCONV_STEP_DW_BWD = 16,       /* BN2 backward + depthwise dgrad/wgrad + Swish' + BN1 partials */
    MBCONV_STEP_DW_WGRAD_REDUCE = 17,  /* sum of the filter-gradient partials; with an expansion conv the same
                                          launch also finalises BN1's backward */
    MBCONV_STEP_BN1_BWD_FINALIZE = 18, /* launches nothing (see step 17): a probe on it times an empty event pair */
    MBCONV_STEP_EXPAND_DGRAD = 19,
    MBCONV_STEP_EXPAND_WGRAD = 20, /* and the sums over the splits of both 1x1 weight gradients (and the
                                      projection conv's weight gradient itself, see PROJ_WGRAD) */
    MBCONV_STEP_COUNT = 21
} mbconv_step;

typedef struct {
    int32_t step;      /* mbconv_step to bracket */
    void *start_event; /* hipEvent_t */
    void *stop_event;  /* hipEvent_t */
} mbconv_probe;

/* Same as mbconv_forward / mbconv_backward, plus the probe (NULL = none).  A probe whose step
 * does not occur in the call (e.g. an expansion step when has_expand == 0) records nothing. */
mbconv_status mbconv_forward_probed(const mbconv_desc *desc, const mbconv_params *params,
                                    mbconv_bn_state *running, const void *x, void *out,
                                    void *saved_ws, void *scratch_ws, void *hip_stream,
                                    const mbconv_probe *probe);
mbconv_status mbconv_backward_probed(const mbconv_desc *desc, const mbconv_params *params,
                                     const void *x, const void *dout, const void *saved_ws,
                                     void *scratch_ws, void *dx, mbconv_grads *grads,
                                     void *hip_stream, const mbconv_probe *probe);

mbconv_status mbconv_forward_eval_probed(const mbconv_desc *desc, const mbconv_params *params,
                                         const mbconv_bn_state *running, const void *x, void *out,
                                         void *workspace, void *hip_stream,
                                         const mbconv_probe *probe);

/* Host-only: which arithmetic units serve one step of the launch sequence for this descriptor
 * (for pricing a measured step against the right roofline).  Steps that are not 1x1 convolutions
 * or their gradients run on the vector units.  A 1x1 step reports the matrix-core instruction
 * family of its kernel: fp32 MFMA; bf16 MFMA on bf16-stored operands; or, for fp32 storage on the
 * wide blocks, bf16 MFMA on operands split into three bf16 planes (six MFMAs per product block,
 * fp32 accumulation: six times the arithmetic of one fp32 product at sixteen times the rate).
 * `step` is an mbconv_step; returns MBCONV_EINVAL for a bad descriptor, step or pointer. */
typedef enum mbconv_engine {
    MBCONV_ENGINE_VECTOR = 0,
    MBCONV_ENGINE_MFMA_F32 = 1,
    MBCONV_ENGINE_MFMA_BF16 = 2,
    MBCONV_ENGINE_MFMA_BF16X3 = 3
} mbconv_engine;
mbconv_status mbconv_step_engine(const mbconv_desc *desc, int32_t step, int32_t *engine);

/* Static string for a status code. */
const char *mbconv_status_string(mbconv_status status);

/* Library version, for the binding's sanity check. */
int32_t mbconv_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MBCONV_H */
