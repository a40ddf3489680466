/*
 * lc.h - C ABI of the locally connected autoencoder kernels for AMD MI355X (gfx950).
 *
 * The library computes, on one GPU, the per-GPU share of the network of Ni et al.,
 * "Large-Scale Deep Learning on the YFCC100M Dataset": layers of untied local receptive
 * fields (Sec. 3.1) trained with the RICA cost of Eq. 1, followed by pooling and local
 * contrast normalisation.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every data pointer is DEVICE memory owned by the caller.  The library allocates
 *    nothing and keeps no pointer after a call returns.  Scratch memory, where an entry
 *    point needs it, is passed in as `ws` / `ws_bytes` (size from lc_workspace_bytes).
 *  - Data pointers must be 16-byte aligned (LC_EALIGN otherwise).
 *  - Activations are [B][H][W][C] with C fastest.  A layer's output is [B][LH][LW][F].
 *    Weights are [LH][LW][K][F], F fastest, with k = (kh*R + kw)*C + c: one K x F matrix
 *    per location.  LH = floor((H-R)/S)+1, LW likewise (valid fields, no padding; trailing
 *    rows/columns that no field covers are ignored by the forward pass and receive zero
 *    from lc_backward_data).
 *  - `dtype` names the storage type of the x / w / dy operands: LC_F32, or LC_BF16 (bf16
 *    operands, fp32 accumulation).  Outputs are always fp32.  Every shape is accepted in
 *    either type.  The bf16 kernels use bf16 matrix instructions wherever the layout allows
 *    whole vectors of bf16 (always for lc_backward_data with R % S == 0, R/S in
 *    {2, 3, 4, 5, 8}, F % 16 == 0 and B > 32; for lc_forward if S*C % 4 == 0, R*C % 4 == 0,
 *    W*C % 4 == 0 and F % 16 == 0; for lc_backward_weights if R*C % 4 == 0 and either
 *    B % 16 == 0 or B <= 128 with S*C % 4 == 0); other shapes widen the bf16 values on their
 *    way in (exactly) and multiply with the fp32 matrix instruction through the same masked
 *    kernels the fp32 path falls back to: the same results either way, at the speed of the
 *    fp32 path with half the operand bytes.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *    only enqueue work; none synchronises.  Arguments are validated on the host before
 *    anything is launched, so every error except LC_EHIP is returned without touching
 *    the GPU.
 *  - Return value: LC_OK (0) or a negative lc_status.  After LC_EHIP,
 *    lc_last_error() gives the HIP error string (thread-local).
 */
#ifndef LC_H_
#define LC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Layer geometry as Sec. 3.1 states it: mini-batch B, input H x W x C, receptive field
 * R x R x C, stride S, F filters per location.  Requires all >= 1, R <= H, R <= W. */
typedef struct {
    int32_t B, H, W, C, R, S, F;
} lc_geom_t;

enum lc_status {
    LC_OK = 0,
    LC_EINVAL = -1,       /* impossible geometry or scalar argument */
    LC_ENULL = -2,        /* a required pointer is NULL */
    LC_EALIGN = -3,       /* a data pointer is not 16-byte aligned */
    LC_EWORKSPACE = -4,   /* ws is NULL or smaller than lc_workspace_bytes() */
    LC_EUNSUPPORTED = -5, /* valid request this build has no kernel for */
    LC_EHIP = -6,         /* a HIP call failed; see lc_last_error() */
    LC_EINTERNAL = -7     /* a launch plan failed the library's own host checks (a bug here, not in the call);
                             nothing was launched; lc_last_error() names the violated condition */
};

enum lc_dtype { LC_F32 = 0, LC_BF16 = 1 };

enum lc_op { LC_OP_FORWARD = 0, LC_OP_BACKWARD_DATA = 1, LC_OP_BACKWARD_WEIGHTS = 2, LC_OP_SAE_STEP = 3 };

/* sae_step flags */
#define LC_SAE_PROJECT_ROWS 1u /* rescale every filter W[l,:,f] to unit L2 norm after the update (constraint of Eq. 1) */
#define LC_SAE_LEARN_ALPHA 2u  /* alpha takes an SGD step too; otherwise it is only read */

/* Host only.  Writes LH, LW, K = R*R*C (any of the three may be NULL).  LC_EINVAL on bad geometry. */
int lc_geom_derive(const lc_geom_t *g, int32_t *LH, int32_t *LW, int32_t *K);

/* Host only.  Bytes of scratch the given lc_op uses for this geometry and dtype (0 = none,
 * then ws may be NULL).  Returns 0 for invalid arguments as well.  LC_OP_SAE_STEP requires its
 * workspace (LC_EWORKSPACE otherwise).  For LC_OP_FORWARD the workspace is optional: a layer with
 * very few fields (the dense last layer of Sec. 3.1 is the one-field case R = H = W) reports a
 * size here, and lc_forward given at least that much cuts the contraction into slices that run
 * side by side; without it the call computes the same result with less of the chip. */
size_t lc_workspace_bytes(const lc_geom_t *g, int op, int dtype);

/* Forward encoding of one layer, the "alpha W x" of Eq. 1 with the geometry of Sec. 3.1:
 *   y[b,i,j,f] = alpha * sum_k w[i,j,k,f] * x[b, i*S+kh, j*S+kw, c]  (+ bias[i,j,f] if bias != NULL)
 * x [B,H,W,C] and w [LH,LW,K,F] in `dtype`; bias [LH,LW,F] fp32 or NULL; y [B,LH,LW,F] fp32, overwritten.
 * ws: optional, see lc_workspace_bytes; its contents are clobbered; must be 16-byte aligned if given. */
int lc_forward(const lc_geom_t *g, const void *x, const void *w, const float *bias, float alpha, float *y,
               int dtype, void *ws, size_t ws_bytes, void *hip_stream);

/* lc_forward with fp32 operands and the scale read from device memory when the kernel runs: alpha_dev points to
 * one float on the device (4-byte aligned).  For a scale that lives on the device because it is being learned
 * there (sae_step's alpha, Eq. 1): a forward-only copy of a layer can follow it without a round trip to the host.
 * Everything else as lc_forward with dtype = LC_F32. */
int lc_forward_dev_scale(const lc_geom_t *g, const float *x, const float *w, const float *bias,
                         const float *alpha_dev, float *y, void *ws, size_t ws_bytes, void *hip_stream);

/* Reconstruction through the transposed filters, the "W^T (.)" of Eq. 1 (also the gradient of
 * lc_forward with respect to x for alpha = 1):
 *   dx[b,p,q,c] = sum over locations (i,j) whose field contains (p,q), sum_f w[i,j,k,f] * dy[b,i,j,f]
 * dy [B,LH,LW,F], w in `dtype`; dx [B,H,W,C] fp32, overwritten everywhere (zero where no field reaches).
 * Deterministic: no atomics. */
int lc_backward_data(const lc_geom_t *g, const void *dy, const void *w, float *dx, int dtype, void *ws,
                     size_t ws_bytes, void *hip_stream);

/* Weight gradient of Eq. 1's terms with respect to the untied filters:
 *   dw[i,j,k,f] = beta * dw[i,j,k,f] + sum_b x[b, i*S+kh, j*S+kw, c] * dy[b,i,j,f]
 * beta must be 0 (dw is overwritten, never read) or 1 (accumulate).  x, dy in `dtype`; dw fp32. */
int lc_backward_weights(const lc_geom_t *g, const void *x, const void *dy, float beta, float *dw, int dtype,
                        void *ws, size_t ws_bytes, void *hip_stream);

/* L2 pooling (not part of the paper's network, Sec. 3.1 leaves pooling out; provided because the
 * benchmark workloads chain it after each layer):
 *   y[b,i,j,c] = sqrt(eps + sum_{p,q<ksize} x[b, i*stride+p, j*stride+q, c]^2), no padding,
 * x [B,H,W,C] -> y [B,Ho,Wo,C], Ho = floor((H-ksize)/stride)+1.  fp32.  1 <= ksize <= min(H,W), eps >= 0. */
int l2pool_fwd(const float *x, float *y, int32_t B, int32_t H, int32_t W, int32_t C, int32_t ksize,
               int32_t stride, float eps, void *hip_stream);

/* Gradient of l2pool_fwd: dx[q] = x[q] * sum over windows containing q of dy/y.  dx [B,H,W,C] overwritten. */
int l2pool_bwd(const float *x, const float *y, const float *dy, float *dx, int32_t B, int32_t H, int32_t W,
               int32_t C, int32_t ksize, int32_t stride, void *hip_stream);

/* Local contrast normalisation, applied after each layer (Sec. 3.1 names it without defining it;
 * this is Gaussian-windowed local standardisation with statistics pooled over all channels):
 *   g[p] ~ exp(-p^2 / (2 gauss_sigma^2)), p = -(ksize-1)/2 .. (ksize-1)/2, window w[p,q] = g[p] g[q];
 *   mu = weighted mean of x over the window and all C channels, m2 the same for x^2 (window truncated
 *   at the border and its weights renormalised); rstd = 1/sqrt(max(m2 - mu^2, 0) + eps);
 *   y[b,i,j,c] = (x[b,i,j,c] - mu[b,i,j]) * rstd[b,i,j].
 * y [B,H,W,C]; mu, rstd [B,H,W] are outputs kept for lcn_bwd.  ksize odd, 1 <= ksize <= 15. */
int lcn_fwd(const float *x, float *y, float *mu, float *rstd, int32_t B, int32_t H, int32_t W, int32_t C,
            int32_t ksize, float gauss_sigma, float eps, void *hip_stream);

/* l2pool_fwd followed by lcn_fwd of its result, as one call (the order the workloads chain them after each
 * layer, Sec. 3.1): p = l2pool_fwd(x), then y, mu, rstd = lcn_fwd(p).  x [B,H,W,C]; p and y [B,Ho,Wo,C];
 * mu, rstd [B,Ho,Wo]; all four are outputs (p is what l2pool_bwd and lcn_bwd read later).  Results are those of the
 * two calls up to fp32 rounding order.  3x3 windows at stride 1 over 8, 16, 32 or 64 channels run as one kernel
 * that never reads p back; other shapes run the two kernels one after the other.  Arguments as in the two calls. */
int l2pool_lcn_fwd(const float *x, float *p, float *y, float *mu, float *rstd, int32_t B, int32_t H, int32_t W,
                   int32_t C, int32_t pool_ksize, int32_t pool_stride, float pool_eps, int32_t lcn_ksize,
                   float gauss_sigma, float lcn_eps, void *hip_stream);

/* Gradient of l2pool_lcn_fwd with respect to x, as one call: dp = lcn_bwd(p, mu, rstd, dy), dx = l2pool_bwd(x, p, dp).
 * x [B,H,W,C] is the pooling input, p, mu, rstd what l2pool_lcn_fwd left, dy [B,Ho,Wo,C] the gradient with respect
 * to its y.  scratch [B,Ho,Wo,C] (fp32, 16-byte aligned, caller-owned) holds the intermediate: dp, or dp / p where the
 * kernels hand that over instead (the pooling gradient then reads one array less); its contents after the call are
 * unspecified.  dx [B,H,W,C] is overwritten.  Results are those of the two calls up to fp32 rounding order. */
int lcn_l2pool_bwd(const float *x, const float *p, const float *mu, const float *rstd, const float *dy,
                   float *scratch, float *dx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t pool_ksize,
                   int32_t pool_stride, int32_t lcn_ksize, float gauss_sigma, void *hip_stream);

/* Gradient of lcn_fwd with respect to x, given the saved mu and rstd (the clamp of the variance at zero is
 * taken as inactive).  dx [B,H,W,C] overwritten. */
int lcn_bwd(const float *x, const float *mu, const float *rstd, const float *dy, float *dx, int32_t B,
            int32_t H, int32_t W, int32_t C, int32_t ksize, float gauss_sigma, void *hip_stream);

/* Variants of lcn_fwd / lcn_bwd (Sec. 3.1 names LCN and gives no formula, so the common published forms are
 * offered beside the default).  flags = 0 is lcn_fwd itself; the bits combine freely:
 *   LCN_PER_CHANNEL  statistics per channel: the window runs over space only, and mu, rstd are [B,H,W,C];
 *   LCN_ZERO_PAD     pixels outside the image count as zeros and the window weights keep their full-window
 *                    normalisation (no renormalisation of the truncated window at the border);
 *   LCN_TWO_STAGE    subtractive then divisive stage: v = x - mean_w(x), y = v / sqrt(mean_w(v^2) + eps), where
 *                    mean_w is the Gaussian-window mean of lcn_fwd and mean_w(v^2) takes every neighbour's own v.
 * mu, rstd ([B,H,W], or [B,H,W,C] with LCN_PER_CHANNEL) hold the subtracted mean and the factor y = (x - mu) rstd.
 * lcn_variant_bwd overwrites dx [B,H,W,C] (which must not alias x or dy); with LCN_TWO_STAGE it needs
 * lcn_variant_workspace_bytes() of scratch (LC_EWORKSPACE otherwise), 0 bytes for the one-stage forms.
 * ksize odd, 1 <= ksize <= 15; unknown flag bits give LC_EINVAL. */
#define LCN_PER_CHANNEL 1u
#define LCN_ZERO_PAD 2u
#define LCN_TWO_STAGE 4u
size_t lcn_variant_workspace_bytes(int32_t B, int32_t H, int32_t W, int32_t C, uint32_t flags);
int lcn_variant_fwd(const float *x, float *y, float *mu, float *rstd, int32_t B, int32_t H, int32_t W, int32_t C,
                    int32_t ksize, float gauss_sigma, float eps, uint32_t flags, void *hip_stream);
int lcn_variant_bwd(const float *x, const float *mu, const float *rstd, const float *dy, float *dx, int32_t B,
                    int32_t H, int32_t W, int32_t C, int32_t ksize, float gauss_sigma, uint32_t flags, void *ws,
                    size_t ws_bytes, void *hip_stream);

/* lcn_variant_bwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments, checks and results as
 * lcn_variant_bwd, minus ws / ws_bytes: the scratch of the two-stage gradient lives in a device array inside the
 * library, LCN_STATIC_SCRATCH_BYTES long, that every GPU the library runs on holds until the process ends.  The
 * call allocates and frees nothing.  A map whose lcn_variant_workspace_bytes() exceeds that size is refused with
 * LC_EWORKSPACE (lc_last_error() says why) before anything is launched.  All calls on one GPU share that GPU's
 * array: two calls that overlap in time on one GPU (different streams or threads) race on it; calls on one stream,
 * or ordered by events, do not.  The first call on a device looks the array's address up (LC_EHIP if that fails). */
#define LCN_STATIC_SCRATCH_BYTES (32u << 20)
int lcn_variant_bwd_static(const float *x, const float *mu, const float *rstd, const float *dy, float *dx, int32_t B,
                           int32_t H, int32_t W, int32_t C, int32_t ksize, float gauss_sigma, uint32_t flags,
                           void *hip_stream);

/* One SGD step on the RICA cost of Eq. 1 for one layer (fp32):
 *   h = alpha W x;  xh = W^T h + b;  J = (1/B) [ sum (xh - x)^2 + lambda * sum sqrt(h^2 + eps_sparse) ]
 *   w -= lr dJ/dw (both uses of the tied weights);  b -= lr dJ/db;  alpha -= lr dJ/dalpha if LC_SAE_LEARN_ALPHA;
 *   then, if LC_SAE_PROJECT_ROWS, every filter w[l,:,f] is rescaled to unit L2 norm.
 * x [B,H,W,C] read only; w [LH,LW,K,F], b [H,W,C] and the device scalar alpha are updated in place;
 * h_out (NULL or [B,LH,LW,F]) receives h computed with the weights from before the update;
 * cost_out is a device scalar that receives J.  Scratch: lc_workspace_bytes(g, LC_OP_SAE_STEP, LC_F32).
 * Preconditions the host cannot check (alpha lives on the device): with LC_SAE_LEARN_ALPHA alpha must be
 * non-zero, because its gradient sum (W x) * dJ/dh is formed as (1/alpha) sum h * dJ/dh; with alpha = 0 the
 * encoder is dead anyway (h = 0 for every input) and the step leaves alpha at NaN.  With LC_SAE_PROJECT_ROWS a
 * filter whose updated values are all exactly zero has no direction and is left as it is (zeros).  With
 * eps_sparse = 0 the sparsity term is |h|, whose gradient at h = 0 is taken as 0. */
int sae_step(const lc_geom_t *g, const float *x, float *w, float *b, float *alpha, float lambda,
             float eps_sparse, float lr, uint32_t flags, float *h_out, float *cost_out, void *ws,
             size_t ws_bytes, void *hip_stream);

/* Thread-local description of the last LC_EHIP on this thread ("" if none). */
const char *lc_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LC_H_ */
