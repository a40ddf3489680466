// sae_step: one SGD step on the RICA cost of Eq. 1 for one layer of untied receptive fields.
//
//   h  = alpha W x                      (lc_forward)
//   xh = W^T h + b, r = xh - x          (lc_backward_data, then the residual kernel below)
//   J  = (1/B) [ sum r^2 + lambda sum sqrt(h^2 + eps) ]
//   u  = 2 r / B,  db = sum_b u
//   gh = W u + (lambda/B) h / sqrt(h^2+eps)          (lc_forward, then the sparsity kernel below)
//   W <- W - lr [ patch(u) h^T + patch(x) (alpha gh)^T ]   (one weight-gradient kernel over both pairs,
//                                                          the update fused into its epilogue)
// The sparsity term needs no second pass over the data (Sec. 3.1): its gradient is an elementwise
// function of h that is added to W u in place.
#include "lc_common.hpp"

namespace lc {

namespace {

constexpr int kPartials = 1024;     // upper bound of the scalar residual pass's partial sums
constexpr int kSparsityThreads = 1024;
constexpr int kSparsityBlocks = 256;   // one workgroup per compute unit: the ticket counter sees few arrivals
constexpr int kPartialsMax = 65536;  // upper bound of the residual pass's partial sums

__device__ __forceinline__ float block_sum(float v, float *sh) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) sh[wave] = v;
    __syncthreads();
    float t = 0.f;
    if (threadIdx.x == 0)
        for (int i = 0; i < (int)(blockDim.x >> 6); ++i) t += sh[i];
    __syncthreads();
    return t;  // valid in thread 0
}

// r = xh + b - x;  u = (2/B) r (written over xh);  part[block] = sum r^2;  dbp[chunk][e] = sum over the
// chunk's images of u.  Grid: x over image elements (float4 per thread), y over chunks of the batch.  The loads of
// four images are in flight together.  Block (0,0) also clears the ticket counter of the sparsity pass.
__global__ __launch_bounds__(256) void sae_residual_kernel(float *__restrict__ xh_u, const float *__restrict__ x,
                                                           const float *__restrict__ b, int B, int img4, int bchunk,
                                                           float *__restrict__ dbp, float *__restrict__ part,
                                                           unsigned *__restrict__ ticket) {
    __shared__ float sh[4];
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *ticket = 0u;
    const int e = blockIdx.x * 256 + threadIdx.x;
    float sq = 0.f;
    if (e < img4) {
        const f32x4 be = ((const f32x4 *)b)[e];
        const float scale = 2.0f / (float)B;
        f32x4 db = (f32x4){0.f, 0.f, 0.f, 0.f};
        const int n0 = blockIdx.y * bchunk, n1 = min(B, n0 + bchunk);
        int n = n0;
        for (; n + 4 <= n1; n += 4) {
            f32x4 a[4], c[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const size_t o = (size_t)(n + t) * img4 + e;
                a[t] = ((const f32x4 *)xh_u)[o];
                c[t] = ((const f32x4 *)x)[o];
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const f32x4 r = a[t] + be - c[t];
                sq += (r[0] * r[0] + r[1] * r[1]) + (r[2] * r[2] + r[3] * r[3]);
                const f32x4 u = scale * r;
                ((f32x4 *)xh_u)[(size_t)(n + t) * img4 + e] = u;
                db += u;
            }
        }
        for (; n < n1; ++n) {
            const size_t o = (size_t)n * img4 + e;
            const f32x4 r = ((const f32x4 *)xh_u)[o] + be - ((const f32x4 *)x)[o];
            sq += (r[0] * r[0] + r[1] * r[1]) + (r[2] * r[2] + r[3] * r[3]);
            const f32x4 u = scale * r;
            ((f32x4 *)xh_u)[o] = u;
            db += u;
        }
        ((f32x4 *)dbp)[(size_t)blockIdx.y * img4 + e] = db;
    }
    const float t = block_sum(sq, sh);
    if (threadIdx.x == 0) part[blockIdx.y * gridDim.x + blockIdx.x] = t;
}

// Same pass for images whose element count is not a multiple of 4: one thread per image element, looping
// over the whole batch; b is updated in place.
__global__ __launch_bounds__(256) void sae_residual_scalar_kernel(float *__restrict__ xh_u,
                                                                  const float *__restrict__ x, float *__restrict__ b,
                                                                  int B, int img, float lr, float *__restrict__ part,
                                                                  unsigned *__restrict__ ticket) {
    __shared__ float sh[4];
    if (blockIdx.x == 0 && threadIdx.x == 0) *ticket = 0u;
    float sq = 0.f;
    for (int e = blockIdx.x * 256 + threadIdx.x; e < img; e += gridDim.x * 256) {
        const float be = b[e];
        const float scale = 2.0f / (float)B;
        float db = 0.f;
        for (int n = 0; n < B; ++n) {
            const size_t o = (size_t)n * img + e;
            const float r = xh_u[o] + be - x[o];
            sq += r * r;
            const float u = scale * r;
            xh_u[o] = u;
            db += u;
        }
        b[e] = be - lr * db;
    }
    const float t = block_sum(sq, sh);
    if (threadIdx.x == 0) part[blockIdx.x] = t;
}

// What the last workgroup of the sparsity pass does with the partial sums of a step.
struct SaeTail {
    unsigned *ticket;          // cleared by the residual pass of the same step
    const float *part_r;       // partial sums of r^2
    int n_r;
    float lambda, lr;
    int B, learn_alpha;
    float *alpha_dev, *cost_out;
    float *bias;               // b -= lr * sum over the batch chunks of dbp, by the workgroups behind the first n_s
    const float *dbp;
    int img, nchunk;
};

// Workgroups [0, n_s):  s = sqrt(h^2+eps);  gh <- alpha * (gh + (lambda/B) h / s);  part_s[block] = sum s;
// part_hg[block] = sum h * gh_before_alpha; four values per lane and four vectors in flight.
// Workgroups [n_s, ...): b -= lr * sum over the batch chunks of dbp, in a fixed order (b is not read any more after
// the residual pass).
// The workgroup of the first n_s that finishes last (a ticket counter: the only atomic of the step, it orders
// nothing but who does the summing) adds the partial sums in a fixed order: cost = (sum r^2 + lambda sum s) / B and
// optionally alpha -= lr * (sum h*gh) / alpha (d h / d alpha = h / alpha); every other workgroup has read alpha by
// then.
__global__ __launch_bounds__(kSparsityThreads) void sae_sparsity_kernel(const float *__restrict__ h, float *__restrict__ gh,
                                                           float lam_over_b, float eps, long long n, int n_s,
                                                           float *__restrict__ part_s, float *__restrict__ part_hg,
                                                           SaeTail tl) {
    __shared__ float sh[kSparsityThreads / 64];
    __shared__ unsigned last;
    if ((int)blockIdx.x >= n_s) {
        const int e = ((int)blockIdx.x - n_s) * kSparsityThreads + threadIdx.x;
        if (e >= tl.img) return;
        float s = 0.f;
        for (int c = 0; c < tl.nchunk; ++c) s += tl.dbp[(size_t)c * tl.img + e];
        tl.bias[e] -= tl.lr * s;
        return;
    }
    const float alpha = *tl.alpha_dev;
    float ss = 0.f, hg = 0.f;
    // s = v * rsq(v) with v = h^2 + eps and h / s = h * rsq(v): one reciprocal square root (1 ulp) instead of a
    // correctly rounded square root and a division, which together cost some forty instructions per value
    auto one = [&](float hv, float gv) {
        const float v = hv * hv + eps;
        const float r = v > 0.f ? __builtin_amdgcn_rsqf(v) : 0.f;     // eps = 0 and h = 0: gradient of |h| taken as 0
        const float g = gv + lam_over_b * (hv * r);
        ss += v * r;
        hg += hv * g;
        return alpha * g;
    };
    constexpr int U = 4;    // vectors of h and of gh in flight per lane
    const long long nv = n / 4, stride = (long long)n_s * kSparsityThreads;
    long long e = (long long)blockIdx.x * kSparsityThreads + threadIdx.x;
    for (; e < nv; e += U * stride) {
        f32x4 hv[U], gv[U];
#pragma unroll
        for (int j = 0; j < U; ++j)
            if (e + j * stride < nv) {
                hv[j] = ((const f32x4 *)h)[e + j * stride];
                gv[j] = ((const f32x4 *)gh)[e + j * stride];
            }
#pragma unroll
        for (int j = 0; j < U; ++j)
            if (e + j * stride < nv) {
                f32x4 o;
#pragma unroll
                for (int c = 0; c < 4; ++c) o[c] = one(hv[j][c], gv[j][c]);
                ((f32x4 *)gh)[e + j * stride] = o;
            }
    }
    if (blockIdx.x == 0 && (long long)threadIdx.x < n - 4 * nv) {       // up to three values behind the last vector
        const long long t = 4 * nv + threadIdx.x;
        gh[t] = one(h[t], gh[t]);
    }
    const float t0 = block_sum(ss, sh);
    const float t1 = block_sum(hg, sh);
    if (threadIdx.x == 0) {
        // The partial sums and the ticket go through agent-scope accesses, which no XCD's L2 keeps to itself, and
        // the ticket is taken only once the two stores have been acknowledged; a release fence here would make
        // every workgroup write back the whole L2 (measured: the kernel four times as long).
        __hip_atomic_store(part_s + blockIdx.x, t0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(part_hg + blockIdx.x, t1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const unsigned k = __hip_atomic_fetch_add(tl.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        last = (k == (unsigned)n_s - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!last) return;
    // every other workgroup's sums were acknowledged before its ticket; part_r comes from an earlier kernel
    float a = 0.f, b = 0.f, c = 0.f;
    for (int i = threadIdx.x; i < tl.n_r; i += kSparsityThreads) a += tl.part_r[i];
    for (int i = threadIdx.x; i < n_s; i += kSparsityThreads) {
        b += __hip_atomic_load(part_s + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        c += __hip_atomic_load(part_hg + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const float ta = block_sum(a, sh), tb = block_sum(b, sh), tc = block_sum(c, sh);
    if (threadIdx.x == 0) {
        *tl.cost_out = (ta + tl.lambda * tb) / (float)tl.B;
        if (tl.learn_alpha) *tl.alpha_dev = alpha - tl.lr * tc / alpha;
    }
}

// Projection onto the constraint of Eq. 1 (every filter w[l,:,f] of unit Euclidean norm) in two small passes behind
// the fused update, whose epilogue already left per-block sums of squares of the updated weights:
//   inv[l,f] = 1 / sqrt(sum over the k blocks of ssq[l,kb,f])   (fixed order: deterministic);
//   w[l,k,f] *= inv[l,f]                                         (one read and one write of w, any number of fields).
// A filter that is all zeros has no direction: it is left as it is (inv = 0 avoids 0 * inf).
__global__ __launch_bounds__(256) void sae_row_norm_kernel(const float *__restrict__ ssq, int kblocks, int F,
                                                           long long LF, float *__restrict__ inv) {
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;     // e = l * F + f
    if (e >= LF) return;
    const long long l = e / F;
    const int f = (int)(e - l * F);
    const float *p = ssq + (size_t)l * kblocks * F + f;
    float t = 0.f;
    for (int kb = 0; kb < kblocks; ++kb) t += p[(size_t)kb * F];
    inv[e] = t > 0.f ? 1.0f / sqrtf(t) : 0.f;
}

template <int V>
__global__ __launch_bounds__(256) void sae_rescale_kernel(float *__restrict__ w, const float *__restrict__ inv, int F,
                                                          long long KF, long long n) {
    typedef typename FVec<V>::T VT;
    const long long nv = n / V;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < nv; e += (long long)gridDim.x * 256) {
        const long long o = e * V, l = o / KF;
        const int f = (int)(o % F);
        VT v = ((const VT *)w)[e];
        const VT s = *(const VT *)(inv + l * F + f);
        ((VT *)w)[e] = v * s;
    }
}

}  // namespace

static size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

// the batch is cut into at most kBatchChunks chunks for the residual pass (more workgroups in flight)
constexpr int kBatchChunks = 16;

size_t sae_workspace_bytes(const Geom &g) {
    const size_t nh = (size_t)g.B * g.L * g.F, nx = (size_t)g.B * g.H * g.W * g.C;
    const size_t img = (size_t)g.H * g.W * g.C;
    return 2 * align256(nh * 4) + align256(nx * 4) + align256(kBatchChunks * img * 4) +
           3 * align256(kPartialsMax * 4) +
           // projection: per-block sums of squares of the updated weights, and the filters' inverse norms
           align256((size_t)g.L * backward_weights_max_kblocks(g) * g.F * 4) + align256((size_t)g.L * g.F * 4) +
           // the slices of lc_forward on a layer with very few fields (0 otherwise)
           align256(forward_wide_workspace_bytes(g));
}

int launch_sae_step(const Geom &g, const float *x, float *w, float *b, float *alpha, float lambda, float eps_sparse,
                    float lr, uint32_t flags, float *h_out, float *cost_out, void *ws, hipStream_t s) {
    const size_t nh = (size_t)g.B * g.L * g.F, nx = (size_t)g.B * g.H * g.W * g.C;
    const int img = g.H * g.W * g.C;
    char *p = (char *)ws;
    float *h_ws = (float *)p; p += align256(nh * 4);
    float *gh = (float *)p;   p += align256(nh * 4);
    float *u = (float *)p;    p += align256(nx * 4);
    float *dbp = (float *)p;  p += align256((size_t)kBatchChunks * img * 4);
    float *part_r = (float *)p; p += align256(kPartialsMax * 4);
    float *part_s = (float *)p; p += align256(kPartialsMax * 4);
    float *part_hg = (float *)p; p += align256(kPartialsMax * 4);
    unsigned *ticket = (unsigned *)(part_hg + kSparsityBlocks);     // behind the sums this array ever holds
    float *ssq = (float *)p;  p += align256((size_t)g.L * backward_weights_max_kblocks(g) * g.F * 4);
    float *inv = (float *)p;  p += align256((size_t)g.L * g.F * 4);
    void *fwd_ws = p;
    const size_t fwd_ws_bytes = forward_wide_workspace_bytes(g);
    float *h = h_out ? h_out : h_ws;
    const bool project = flags & LC_SAE_PROJECT_ROWS;

    int rc;
    if ((rc = launch_forward_f32(g, x, w, nullptr, 1.f, alpha, h, s, fwd_ws, fwd_ws_bytes)) != LC_OK) return rc;
    if ((rc = launch_backward_data_f32(g, h, w, u, s)) != LC_OK) return rc;
    int n_r, bias_chunks = 0;     // bias_chunks > 0: the b update waits for the sparsity pass
    if ((img & 3) == 0 && (img / 4 + 255) / 256 * kBatchChunks <= kPartialsMax) {
        const int img4 = img / 4, gx = (img4 + 255) / 256;
        const int nchunk = g.B < kBatchChunks ? g.B : kBatchChunks, bchunk = (g.B + nchunk - 1) / nchunk;
        const int gy = (g.B + bchunk - 1) / bchunk;
        const LaunchPlan plan = make_plan("sae_residual", {4}, {img4, bchunk}, dim3(gx, gy), 256, 0);
        LC_PLAN_REQUIRE(plan, gx * gy <= kPartialsMax && gy <= kBatchChunks && (long long)gy * bchunk >= g.B);
        LC_LAUNCH(plan, "sae_step residual launch", sae_residual_kernel, s, u, x, b, g.B, img4, bchunk, dbp, part_r,
                  ticket);
        bias_chunks = gy;
        n_r = gx * gy;
    } else {
        n_r = (int)((img + 255) / 256 < kPartials ? (img + 255) / 256 : kPartials);
        const LaunchPlan plan = make_plan("sae_residual", {1}, {img}, dim3(n_r), 256, 0);
        LC_LAUNCH(plan, "sae_step residual launch", sae_residual_scalar_kernel, s, u, x, b, g.B, img, lr, part_r,
                  ticket);
    }
    if ((rc = launch_forward_f32(g, u, w, nullptr, 1.f, nullptr, gh, s, fwd_ws, fwd_ws_bytes)) != LC_OK) return rc;
    // four values per lane, four vectors per trip: at most kSparsityBlocks workgroups, at least one
    const size_t nsw = (nh / 4 + 4 * kSparsityThreads - 1) / (4 * kSparsityThreads);
    const int n_s = (int)(nsw < 1 ? 1 : nsw < (size_t)kSparsityBlocks ? nsw : kSparsityBlocks);
    {
        // the workgroups behind the first n_s update b; the last of the first n_s to finish writes the cost
        const int bias_blocks = bias_chunks > 0 ? (img + kSparsityThreads - 1) / kSparsityThreads : 0;
        const LaunchPlan plan = make_plan("sae_sparsity", {}, {n_s, n_r, bias_chunks}, dim3(n_s + bias_blocks),
                                          kSparsityThreads, 0);
        LC_PLAN_REQUIRE(plan, n_s >= 1 && n_s <= kSparsityBlocks && n_r <= kPartialsMax);
        const SaeTail tl = {ticket, part_r, n_r, lambda, lr, g.B, (flags & LC_SAE_LEARN_ALPHA) ? 1 : 0, alpha, cost_out,
                            b, dbp, img, bias_chunks};
        LC_LAUNCH(plan, "sae_step sparsity launch", sae_sparsity_kernel, s, h, gh, lambda / (float)g.B, eps_sparse,
                  (long long)nh, n_s, part_s, part_hg, tl);
    }
    // w <- w - lr * ( patch(u) h^T + patch(x) (alpha gh)^T ), with the sums of squares of the new weights on the side
    int kblocks = 0;
    if ((rc = launch_backward_weights_f32(g, u, h, x, gh, 1.f, -lr, w, s, project ? ssq : nullptr, &kblocks)) != LC_OK)
        return rc;
    if (project) {
        const long long LF = (long long)g.L * g.F, KF = (long long)g.K * g.F, nw = (long long)g.L * KF;
        const LaunchPlan pn = make_plan("sae_row_norm", {}, {kblocks}, dim3((unsigned)((LF + 255) / 256)), 256, 0);
        LC_PLAN_REQUIRE(pn, kblocks >= 1 && kblocks <= backward_weights_max_kblocks(g));
        LC_LAUNCH(pn, "sae_step projection launch", sae_row_norm_kernel, s, ssq, kblocks, g.F, LF, inv);
        // vectors of four filters where a row of w is made of them (a vector then never straddles two filters' rows)
        const int V = g.F % 4 == 0 ? 4 : 1;
        const long long nv = nw / V;
        const unsigned blocks = (unsigned)(nv / 256 + 1 < 256 * 32 ? nv / 256 + 1 : 256 * 32);
        const LaunchPlan pr = make_plan("sae_rescale", {V}, {}, dim3(blocks), 256, 0);
        if (V == 4)
            LC_LAUNCH(pr, "sae_step projection launch", sae_rescale_kernel<4>, s, w, inv, g.F, KF, nw);
        else
            LC_LAUNCH(pr, "sae_step projection launch", sae_rescale_kernel<1>, s, w, inv, g.F, KF, nw);
    }
    return LC_OK;
}

}  // namespace lc
