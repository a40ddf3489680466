// C ABI of the library: argument validation on the host, then dispatch to the kernel launchers.
#include <stdio.h>
#include <string.h>

#include <map>
#include <mutex>
#include <utility>
#include <vector>

#include "lc_common.hpp"

namespace lc {

static thread_local char g_err[256] = "";

void set_hip_error(hipError_t e, const char *where) {
    snprintf(g_err, sizeof(g_err), "%s: %s", where, hipGetErrorString(e));
}

void set_error_text(const char *text) { snprintf(g_err, sizeof(g_err), "%s", text); }

// ---------------------------------------------------------------------------------------------
// Launch plans: see lc_common.hpp.
static thread_local std::vector<LaunchPlan> *g_capture = nullptr;

bool plan_capture() { return g_capture != nullptr; }
void plan_capture_add(const LaunchPlan &p) { g_capture->push_back(p); }

LaunchPlan make_plan(const char *kernel, std::initializer_list<int> tparam, std::initializer_list<int> arg, dim3 grid,
                     unsigned block, size_t lds_bytes) {
    LaunchPlan p;
    memset(&p, 0, sizeof(p));
    snprintf(p.kernel, sizeof(p.kernel), "%s", kernel);
    int n = 0;
    for (int v : tparam)
        if (n < 12) p.tparam[n++] = v;
    n = 0;
    for (int v : arg)
        if (n < 12) p.arg[n++] = v;
    p.grid[0] = grid.x; p.grid[1] = grid.y; p.grid[2] = grid.z;
    p.block = block;
    p.lds_bytes = lds_bytes;
    return p;
}

int plan_fail(const LaunchPlan &p, const char *what) {
    snprintf(g_err, sizeof(g_err), "%s: launch plan violates: %s", p.kernel, what);
    return LC_EINTERNAL;
}

int check_launch_shape(const LaunchPlan &p) {
    LC_PLAN_REQUIRE(p, p.grid[0] >= 1 && p.grid[0] <= 0x7fffffffu);
    LC_PLAN_REQUIRE(p, p.grid[1] >= 1 && p.grid[1] <= 65535u && p.grid[2] >= 1 && p.grid[2] <= 65535u);
    LC_PLAN_REQUIRE(p, p.block >= 64 && p.block <= 1024 && p.block % 64 == 0);
    LC_PLAN_REQUIRE(p, p.lds_bytes <= 160u * 1024u);
    return LC_OK;
}

// Kernels that stage more than 48 KB need their dynamic LDS limit raised; the attribute is set once per
// (kernel, device) and remembered, so a launch costs a table lookup instead of a runtime call.
int allow_dynamic_lds(const void *kernel, size_t bytes, const char *where) {
    if (bytes <= 48 * 1024) return LC_OK;
    static std::mutex mu;
    static std::map<std::pair<const void *, int>, size_t> granted;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_hip_error(e, where); return LC_EHIP; }
    std::lock_guard<std::mutex> lock(mu);
    size_t &have = granted[{kernel, dev}];
    if (bytes <= have) return LC_OK;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) { set_hip_error(e, where); return LC_EHIP; }
    have = bytes;
    return LC_OK;
}

static inline bool aligned16(const void *p) { return ptr_aligned16(p); }

}  // namespace lc

using namespace lc;

#define LC_REQUIRE_PTR(p)                 \
    do {                                  \
        if (!(p)) return LC_ENULL;        \
    } while (0)
#define LC_REQUIRE_ALIGNED(p)                 \
    do {                                      \
        if (!aligned16(p)) return LC_EALIGN;  \
    } while (0)

extern "C" {

int lc_geom_derive(const lc_geom_t *g, int32_t *LH, int32_t *LW, int32_t *K) {
    Geom q;
    if (!make_geom(g, &q)) return LC_EINVAL;
    if (LH) *LH = q.LH;
    if (LW) *LW = q.LW;
    if (K) *K = q.K;
    return LC_OK;
}

size_t lc_workspace_bytes(const lc_geom_t *g, int op, int dtype) {
    Geom q;
    if (!make_geom(g, &q)) return 0;
    if (dtype != LC_F32 && dtype != LC_BF16) return 0;
    if (op == LC_OP_SAE_STEP) return sae_workspace_bytes(q);
    if (op == LC_OP_FORWARD && dtype == LC_F32) return forward_wide_workspace_bytes(q);
    return 0;
}

const char *lc_last_error(void) { return g_err; }

int lc_forward(const lc_geom_t *g, const void *x, const void *w, const float *bias, float alpha, float *y, int dtype,
               void *ws, size_t ws_bytes, void *hip_stream) {
    Geom q;
    if (!make_geom(g, &q)) return LC_EINVAL;
    if (dtype != LC_F32 && dtype != LC_BF16) return LC_EINVAL;
    LC_REQUIRE_PTR(x); LC_REQUIRE_PTR(w); LC_REQUIRE_PTR(y);
    LC_REQUIRE_ALIGNED(ws);
    LC_REQUIRE_ALIGNED(x); LC_REQUIRE_ALIGNED(w); LC_REQUIRE_ALIGNED(y); LC_REQUIRE_ALIGNED(bias);
    if (dtype == LC_BF16) return launch_forward_bf16(q, x, w, bias, alpha, y, (hipStream_t)hip_stream);
    return launch_forward_f32(q, (const float *)x, (const float *)w, bias, alpha, nullptr, y, (hipStream_t)hip_stream, ws,
                              ws_bytes);
}

int lc_forward_dev_scale(const lc_geom_t *g, const float *x, const float *w, const float *bias, const float *alpha_dev,
                         float *y, void *ws, size_t ws_bytes, void *hip_stream) {
    Geom q;
    if (!make_geom(g, &q)) return LC_EINVAL;
    LC_REQUIRE_PTR(x); LC_REQUIRE_PTR(w); LC_REQUIRE_PTR(y); LC_REQUIRE_PTR(alpha_dev);
    LC_REQUIRE_ALIGNED(ws);
    LC_REQUIRE_ALIGNED(x); LC_REQUIRE_ALIGNED(w); LC_REQUIRE_ALIGNED(y); LC_REQUIRE_ALIGNED(bias);
    if ((uintptr_t)alpha_dev & 3u) return LC_EALIGN;
    return launch_forward_f32(q, x, w, bias, 1.f, alpha_dev, y, (hipStream_t)hip_stream, ws, ws_bytes);
}

int lc_backward_data(const lc_geom_t *g, const void *dy, const void *w, float *dx, int dtype, void *ws,
                     size_t ws_bytes, void *hip_stream) {
    (void)ws; (void)ws_bytes;
    Geom q;
    if (!make_geom(g, &q)) return LC_EINVAL;
    if (dtype != LC_F32 && dtype != LC_BF16) return LC_EINVAL;
    LC_REQUIRE_PTR(dy); LC_REQUIRE_PTR(w); LC_REQUIRE_PTR(dx);
    LC_REQUIRE_ALIGNED(dy); LC_REQUIRE_ALIGNED(w); LC_REQUIRE_ALIGNED(dx);
    if (dtype == LC_BF16) return launch_backward_data_bf16(q, dy, w, dx, (hipStream_t)hip_stream);
    return launch_backward_data_f32(q, (const float *)dy, (const float *)w, dx, (hipStream_t)hip_stream);
}

int lc_backward_weights(const lc_geom_t *g, const void *x, const void *dy, float beta, float *dw, int dtype, void *ws,
                        size_t ws_bytes, void *hip_stream) {
    (void)ws; (void)ws_bytes;
    Geom q;
    if (!make_geom(g, &q)) return LC_EINVAL;
    if (dtype != LC_F32 && dtype != LC_BF16) return LC_EINVAL;
    if (!(beta == 0.f || beta == 1.f)) return LC_EINVAL;
    LC_REQUIRE_PTR(x); LC_REQUIRE_PTR(dy); LC_REQUIRE_PTR(dw);
    LC_REQUIRE_ALIGNED(x); LC_REQUIRE_ALIGNED(dy); LC_REQUIRE_ALIGNED(dw);
    if (dtype == LC_BF16) return launch_backward_weights_bf16(q, x, dy, beta, dw, (hipStream_t)hip_stream);
    return launch_backward_weights_f32(q, (const float *)x, (const float *)dy, nullptr, nullptr, beta, 1.f, dw,
                                       (hipStream_t)hip_stream);
}

int lc_plan_query(const lc_geom_t *g, int op, int dtype, lc_launch_t *out, int32_t max_out, int32_t *n_out) {
    Geom q;
    if (!make_geom(g, &q)) return LC_EINVAL;
    if (dtype != LC_F32 && dtype != LC_BF16) return LC_EINVAL;
    if (max_out < 0 || (max_out > 0 && !out) || !n_out) return LC_EINVAL;
    if (op == LC_OP_SAE_STEP && dtype != LC_F32) return LC_EINVAL;
    // never dereferenced: the launchers only do address arithmetic on the host, and nothing is launched
    char *fake = (char *)(uintptr_t)0x100000;
    float *ff = (float *)fake;
    std::vector<LaunchPlan> plans;
    g_capture = &plans;
    int rc = LC_EINVAL;
    const hipStream_t s = nullptr;
    if (op == LC_OP_FORWARD) {
        rc = dtype == LC_BF16 ? launch_forward_bf16(q, fake, fake, nullptr, 1.f, ff, s)
                              : launch_forward_f32(q, ff, ff, nullptr, 1.f, nullptr, ff, s, fake,
                                                   forward_wide_workspace_bytes(q));
    } else if (op == LC_OP_BACKWARD_DATA) {
        rc = dtype == LC_BF16 ? launch_backward_data_bf16(q, fake, fake, ff, s) : launch_backward_data_f32(q, ff, ff, ff, s);
    } else if (op == LC_OP_BACKWARD_WEIGHTS) {
        rc = dtype == LC_BF16 ? launch_backward_weights_bf16(q, fake, fake, 0.f, ff, s)
                              : launch_backward_weights_f32(q, ff, ff, nullptr, nullptr, 0.f, 1.f, ff, s);
    } else if (op == LC_OP_SAE_STEP) {
        rc = launch_sae_step(q, ff, ff, ff, ff, 0.1f, 1e-6f, 1e-3f, LC_SAE_PROJECT_ROWS | LC_SAE_LEARN_ALPHA, ff, ff, fake, s);
    }
    g_capture = nullptr;
    if (rc != LC_OK) return rc;
    *n_out = (int32_t)plans.size();
    for (int32_t k = 0; k < max_out && k < (int32_t)plans.size(); ++k) out[k] = plans[k];
    return LC_OK;
}

static int check_map(int32_t B, int32_t H, int32_t W, int32_t C) { return check_map_dims(B, H, W, C); }

int l2pool_lcn_plan_query(int32_t B, int32_t H, int32_t W, int32_t C, int32_t pool_ksize, int32_t pool_stride,
                          int32_t lcn_ksize, float gauss_sigma, lc_launch_t *out, int32_t max_out, int32_t *n_out) {
    if (check_map(B, H, W, C) != LC_OK) return LC_EINVAL;
    if (pool_ksize < 1 || pool_stride < 1 || pool_ksize > H || pool_ksize > W) return LC_EINVAL;
    if (lcn_ksize < 1 || lcn_ksize > 15 || (lcn_ksize & 1) == 0 || !(gauss_sigma > 0.f)) return LC_EINVAL;
    if (max_out < 0 || (max_out > 0 && !out) || !n_out) return LC_EINVAL;
    *n_out = 0;
    if (pool_ksize != 3 || pool_stride != 1) return LC_OK;
    float *ff = (float *)(uintptr_t)0x100000;      // never dereferenced: nothing is launched
    std::vector<LaunchPlan> plans;
    bool done = false;
    g_capture = &plans;
    const int rc = launch_pool_lcn_fused(ff, ff, ff, ff, ff, B, H, W, C, 1e-6f, lcn_ksize, gauss_sigma, 1e-4f, nullptr, &done);
    g_capture = nullptr;
    if (rc != LC_OK) return rc;
    *n_out = (int32_t)plans.size();
    for (int32_t k = 0; k < max_out && k < (int32_t)plans.size(); ++k) out[k] = plans[k];
    return LC_OK;
}

int l2pool_fwd(const float *x, float *y, int32_t B, int32_t H, int32_t W, int32_t C, int32_t ksize, int32_t stride,
               float eps, void *hip_stream) {
    if (check_map(B, H, W, C) != LC_OK) return LC_EINVAL;
    if (ksize < 1 || stride < 1 || ksize > H || ksize > W || !(eps >= 0.f)) return LC_EINVAL;
    LC_REQUIRE_PTR(x); LC_REQUIRE_PTR(y);
    LC_REQUIRE_ALIGNED(x); LC_REQUIRE_ALIGNED(y);
    return launch_l2pool_fwd(x, y, B, H, W, C, ksize, stride, eps, (hipStream_t)hip_stream);
}

int l2pool_bwd(const float *x, const float *y, const float *dy, float *dx, int32_t B, int32_t H, int32_t W, int32_t C,
               int32_t ksize, int32_t stride, void *hip_stream) {
    if (check_map(B, H, W, C) != LC_OK) return LC_EINVAL;
    if (ksize < 1 || stride < 1 || ksize > H || ksize > W) return LC_EINVAL;
    LC_REQUIRE_PTR(x); LC_REQUIRE_PTR(y); LC_REQUIRE_PTR(dy); LC_REQUIRE_PTR(dx);
    LC_REQUIRE_ALIGNED(x); LC_REQUIRE_ALIGNED(y); LC_REQUIRE_ALIGNED(dy); LC_REQUIRE_ALIGNED(dx);
    return launch_l2pool_bwd(x, y, dy, dx, B, H, W, C, ksize, stride, (hipStream_t)hip_stream);
}

int lcn_fwd(const float *x, float *y, float *mu, float *rstd, int32_t B, int32_t H, int32_t W, int32_t C,
            int32_t ksize, float gauss_sigma, float eps, void *hip_stream) {
    if (check_map(B, H, W, C) != LC_OK) return LC_EINVAL;
    if (ksize < 1 || ksize > 15 || (ksize & 1) == 0 || !(gauss_sigma > 0.f) || !(eps >= 0.f)) return LC_EINVAL;
    LC_REQUIRE_PTR(x); LC_REQUIRE_PTR(y); LC_REQUIRE_PTR(mu); LC_REQUIRE_PTR(rstd);
    LC_REQUIRE_ALIGNED(x); LC_REQUIRE_ALIGNED(y); LC_REQUIRE_ALIGNED(mu); LC_REQUIRE_ALIGNED(rstd);
    return launch_lcn(0, x, nullptr, y, mu, rstd, B, H, W, C, ksize, gauss_sigma, eps, (hipStream_t)hip_stream);
}

int l2pool_lcn_fwd(const float *x, float *p, float *y, float *mu, float *rstd, int32_t B, int32_t H, int32_t W,
                   int32_t C, int32_t pool_ksize, int32_t pool_stride, float pool_eps, int32_t lcn_ksize,
                   float gauss_sigma, float lcn_eps, void *hip_stream) {
    if (check_map(B, H, W, C) != LC_OK) return LC_EINVAL;
    if (pool_ksize < 1 || pool_stride < 1 || pool_ksize > H || pool_ksize > W || !(pool_eps >= 0.f)) return LC_EINVAL;
    if (lcn_ksize < 1 || lcn_ksize > 15 || (lcn_ksize & 1) == 0 || !(gauss_sigma > 0.f) || !(lcn_eps >= 0.f))
        return LC_EINVAL;
    LC_REQUIRE_PTR(x); LC_REQUIRE_PTR(p); LC_REQUIRE_PTR(y); LC_REQUIRE_PTR(mu); LC_REQUIRE_PTR(rstd);
    LC_REQUIRE_ALIGNED(x); LC_REQUIRE_ALIGNED(p); LC_REQUIRE_ALIGNED(y); LC_REQUIRE_ALIGNED(mu); LC_REQUIRE_ALIGNED(rstd);
    hipStream_t s = (hipStream_t)hip_stream;
    if (pool_ksize == 3 && pool_stride == 1) {
        bool done = false;
        const int rc = launch_pool_lcn_fused(x, p, y, mu, rstd, B, H, W, C, pool_eps, lcn_ksize, gauss_sigma, lcn_eps, s,
                                             &done);
        if (done || rc != LC_OK) return rc;
    }
    const int Ho = (H - pool_ksize) / pool_stride + 1, Wo = (W - pool_ksize) / pool_stride + 1;
    if (int rc = launch_l2pool_fwd(x, p, B, H, W, C, pool_ksize, pool_stride, pool_eps, s)) return rc;
    return launch_lcn(0, p, nullptr, y, mu, rstd, B, Ho, Wo, C, lcn_ksize, gauss_sigma, lcn_eps, s);
}

int lcn_l2pool_bwd(const float *x, const float *p, const float *mu, const float *rstd, const float *dy,
                   float *scratch, float *dx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t pool_ksize,
                   int32_t pool_stride, int32_t lcn_ksize, float gauss_sigma, void *hip_stream) {
    if (check_map(B, H, W, C) != LC_OK) return LC_EINVAL;
    if (pool_ksize < 1 || pool_stride < 1 || pool_ksize > H || pool_ksize > W) return LC_EINVAL;
    if (lcn_ksize < 1 || lcn_ksize > 15 || (lcn_ksize & 1) == 0 || !(gauss_sigma > 0.f)) return LC_EINVAL;
    LC_REQUIRE_PTR(x); LC_REQUIRE_PTR(p); LC_REQUIRE_PTR(mu); LC_REQUIRE_PTR(rstd); LC_REQUIRE_PTR(dy);
    LC_REQUIRE_PTR(scratch); LC_REQUIRE_PTR(dx);
    LC_REQUIRE_ALIGNED(x); LC_REQUIRE_ALIGNED(p); LC_REQUIRE_ALIGNED(mu); LC_REQUIRE_ALIGNED(rstd); LC_REQUIRE_ALIGNED(dy);
    LC_REQUIRE_ALIGNED(scratch); LC_REQUIRE_ALIGNED(dx);
    if (scratch == dy || scratch == p || dx == x) return LC_EINVAL;
    return launch_lcn_pool_bwd(x, p, mu, rstd, dy, scratch, dx, B, H, W, C, pool_ksize, pool_stride, lcn_ksize,
                               gauss_sigma, (hipStream_t)hip_stream);
}

int lcn_bwd(const float *x, const float *mu, const float *rstd, const float *dy, float *dx, int32_t B, int32_t H,
            int32_t W, int32_t C, int32_t ksize, float gauss_sigma, void *hip_stream) {
    if (check_map(B, H, W, C) != LC_OK) return LC_EINVAL;
    if (ksize < 1 || ksize > 15 || (ksize & 1) == 0 || !(gauss_sigma > 0.f)) return LC_EINVAL;
    LC_REQUIRE_PTR(x); LC_REQUIRE_PTR(mu); LC_REQUIRE_PTR(rstd); LC_REQUIRE_PTR(dy); LC_REQUIRE_PTR(dx);
    LC_REQUIRE_ALIGNED(x); LC_REQUIRE_ALIGNED(mu); LC_REQUIRE_ALIGNED(rstd); LC_REQUIRE_ALIGNED(dy); LC_REQUIRE_ALIGNED(dx);
    return launch_lcn(1, x, dy, dx, const_cast<float *>(mu), const_cast<float *>(rstd), B, H, W, C, ksize, gauss_sigma,
                      0.f, (hipStream_t)hip_stream);
}

size_t lcn_variant_workspace_bytes(int32_t B, int32_t H, int32_t W, int32_t C, uint32_t flags) {
    if (check_map(B, H, W, C) != LC_OK || (flags & ~7u)) return 0;
    return lc::lcn_variant_scratch_bytes(B, H, W, C, flags);
}

int lcn_variant_fwd(const float *x, float *y, float *mu, float *rstd, int32_t B, int32_t H, int32_t W, int32_t C,
                    int32_t ksize, float gauss_sigma, float eps, uint32_t flags, void *hip_stream) {
    if (check_map(B, H, W, C) != LC_OK || (flags & ~7u)) return LC_EINVAL;
    if (ksize < 1 || ksize > 15 || (ksize & 1) == 0 || !(gauss_sigma > 0.f) || !(eps >= 0.f)) return LC_EINVAL;
    LC_REQUIRE_PTR(x); LC_REQUIRE_PTR(y); LC_REQUIRE_PTR(mu); LC_REQUIRE_PTR(rstd);
    LC_REQUIRE_ALIGNED(x); LC_REQUIRE_ALIGNED(y); LC_REQUIRE_ALIGNED(mu); LC_REQUIRE_ALIGNED(rstd);
    return launch_lcn_variant_fwd(x, y, mu, rstd, B, H, W, C, ksize, gauss_sigma, eps, flags, (hipStream_t)hip_stream);
}

int lcn_variant_bwd(const float *x, const float *mu, const float *rstd, const float *dy, float *dx, int32_t B,
                    int32_t H, int32_t W, int32_t C, int32_t ksize, float gauss_sigma, uint32_t flags, void *ws,
                    size_t ws_bytes, void *hip_stream) {
    if (int rc = check_lcn_variant_bwd_args(x, mu, rstd, dy, dx, B, H, W, C, ksize, gauss_sigma, flags)) return rc;
    if (flags & LCN_TWO_STAGE) {
        if (ws == nullptr || ws_bytes < lc::lcn_variant_scratch_bytes(B, H, W, C, flags)) return LC_EWORKSPACE;
        LC_REQUIRE_ALIGNED(ws);
    }
    return launch_lcn_variant_bwd(x, mu, rstd, dy, dx, B, H, W, C, ksize, gauss_sigma, flags, ws, ws_bytes,
                                  (hipStream_t)hip_stream);
}

int sae_step(const lc_geom_t *g, const float *x, float *w, float *b, float *alpha, float lambda, float eps_sparse,
             float lr, uint32_t flags, float *h_out, float *cost_out, void *ws, size_t ws_bytes, void *hip_stream) {
    Geom q;
    if (!make_geom(g, &q)) return LC_EINVAL;
    if (!(lambda >= 0.f) || !(eps_sparse >= 0.f) || !(lr == lr) || (flags & ~3u)) return LC_EINVAL;
    LC_REQUIRE_PTR(x); LC_REQUIRE_PTR(w); LC_REQUIRE_PTR(b); LC_REQUIRE_PTR(alpha); LC_REQUIRE_PTR(cost_out);
    LC_REQUIRE_ALIGNED(x); LC_REQUIRE_ALIGNED(w); LC_REQUIRE_ALIGNED(b); LC_REQUIRE_ALIGNED(h_out);
    if (((uintptr_t)alpha & 3u) || ((uintptr_t)cost_out & 3u)) return LC_EALIGN;
    if (!ws || ws_bytes < sae_workspace_bytes(q)) return LC_EWORKSPACE;
    LC_REQUIRE_ALIGNED(ws);
    return launch_sae_step(q, x, w, b, alpha, lambda, eps_sparse, lr, flags, h_out, cost_out, ws,
                           (hipStream_t)hip_stream);
}

}  // extern "C"
