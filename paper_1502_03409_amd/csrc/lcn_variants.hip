// Variants of the local contrast normalisation applied after each layer (Sec. 3.1 names LCN without defining it):
// statistics per channel instead of pooled over the channels, zero-padded instead of renormalised borders, and
// the two-stage form (subtract the local mean, then divide by the local root mean square of the result).
//
// Pooled statistics run in the channel-reduction kernels of the default form (pool_lcn.hip).  This file holds the
// per-channel kernel: every element has its own statistics, so a workgroup stages an 8x16 pixel tile, its halo and
// up to 32 channels of the quantity under the window in LDS (as float4 where C % 4 == 0), and each thread forms
// the Gaussian window sums for one pixel and four channels at a time.  Bandwidth-bound: the forward passes read
// the tile once (the centre value is taken from LDS), the halo ring comes from L2.
#include <mutex>

#include "lc_common.hpp"

namespace lc {
namespace {

constexpr int kTileH = 8, kTileW = 16;
constexpr int kMaxK = 15;
constexpr int kLdsTarget = 32 * 1024;   // per workgroup: several workgroups per compute unit hide the load latency

struct Taps { float g[kMaxK]; };

enum : int {
    kFwdOne,    // x -> mu, rstd, y (one stage)
    kMean,      // x -> mu
    kDivide,    // x, mu -> rstd, y = (x - mu) rstd with the window mean of the neighbours' own (x - mu)^2
    kBwdOne,    // one-stage gradient
    kBwdTwoA,   // two-stage gradient up to dv (written to dx) and field = dv / normaliser
    kBwdTwoB    // dx = dv - window sum of field
};

struct Args {
    const float *x, *dy, *mu_in, *rstd_in;
    float *out, *mu_out, *rstd_out, *field;
    int H, W, C, CB, ks, zpad, tiles_w, tiles_per_img, nchunk;
    float eps;
    Taps taps;
};

__device__ __forceinline__ float taps_inside(const Taps &t, int p, int n, int r) {
    float z = 0.f;
    for (int d = -r; d <= r; ++d)
        if (p + d >= 0 && p + d < n) z += t.g[d + r];
    return z;
}

template <int V> struct Pack { float v[V]; };

template <int V> __device__ __forceinline__ Pack<V> load(const float *p) {
    Pack<V> r;
    if constexpr (V == 4) {
        const float4 t = *(const float4 *)p;
        r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
    } else {
        r.v[0] = *p;
    }
    return r;
}

template <int V> __device__ __forceinline__ void store(float *p, const Pack<V> &r) {
    if constexpr (V == 4) *(float4 *)p = make_float4(r.v[0], r.v[1], r.v[2], r.v[3]);
    else *p = r.v[0];
}

// V channels per work item (4 where C % 4 == 0); a.CB channels per workgroup, a multiple of V.
template <int OP, int V>
__global__ __launch_bounds__(256) void lcn_channel_kernel(Args a) {
    extern __shared__ __align__(16) float lds[];
    constexpr bool kTwoMaps = OP == kBwdOne;
    const int r = (a.ks - 1) / 2, hh = kTileH + 2 * r, hw = kTileW + 2 * r, H = a.H, W = a.W, C = a.C;
    const int CBV = a.CB / V;
    float *m1 = lds, *m2 = lds + hh * hw * a.CB;
    const int tid = threadIdx.x;
    int blk = remap_xcd(blockIdx.x, gridDim.x);   // an image's tiles, whose halos overlap, stay in one XCD's L2
    const int chunk = blk % a.nchunk;
    blk /= a.nchunk;
    const int b = blk / a.tiles_per_img, tile = blk - b * a.tiles_per_img;
    const int ti = (tile / a.tiles_w) * kTileH, tj = (tile % a.tiles_w) * kTileW;
    const int c0 = chunk * a.CB, ncv = min(CBV, (C - c0) / V);
    const size_t img = (size_t)b * H * W;
    // window normalisers of the staged rows and columns, once per workgroup (an element's is their product)
    __shared__ float zr[kTileH + kMaxK - 1], zc[kTileW + kMaxK - 1];
    if (tid < hh) zr[tid] = a.zpad ? 1.f : taps_inside(a.taps, ti - r + tid, H, r);
    else if (tid >= 64 && tid < 64 + hw) zc[tid - 64] = a.zpad ? 1.f : taps_inside(a.taps, tj - r + tid - 64, W, r);
    if (OP == kBwdOne || OP == kBwdTwoA) __syncthreads();   // the other passes first use them after phase 1's barrier
    auto norm_at = [&](int row, int col) { return zr[row - ti + r] * zc[col - tj + r]; };

    // phase 1: the quantity under the window for the tile and its halo; zeros outside the image
    for (int idx = tid; idx < hh * hw * CBV; idx += 256) {
        const int hp = idx / CBV, cv = idx - hp * CBV;
        const int hi = hp / hw, hj = hp - hi * hw;
        const int row = ti - r + hi, col = tj - r + hj;
        Pack<V> p1, p2;
#pragma unroll
        for (int k = 0; k < V; ++k) p1.v[k] = p2.v[k] = 0.f;
        if (cv < ncv && row >= 0 && row < H && col >= 0 && col < W) {
            const size_t e = (img + (size_t)row * W + col) * C + c0 + cv * V;
            if (OP == kBwdTwoB) {
                p1 = load<V>(a.field + e);
            } else if (OP == kFwdOne || OP == kMean) {
                p1 = load<V>(a.x + e);
            } else if (OP == kDivide) {
                const Pack<V> xv = load<V>(a.x + e), m = load<V>(a.mu_in + e);
#pragma unroll
                for (int k = 0; k < V; ++k) p1.v[k] = xv.v[k] - m.v[k];
            } else {
                const Pack<V> xv = load<V>(a.x + e), dv = load<V>(a.dy + e), m = load<V>(a.mu_in + e),
                              rs = load<V>(a.rstd_in + e);
                const float iz = 1.f / norm_at(row, col);
#pragma unroll
                for (int k = 0; k < V; ++k) {
                    // gradients of this element's window mean and second moment (or variance), over its normaliser
                    const float bc = rs.v[k] * rs.v[k] * rs.v[k] * dv.v[k] * (xv.v[k] - m.v[k]);
                    if (OP == kBwdOne) {
                        p1.v[k] = (bc * m.v[k] - rs.v[k] * dv.v[k]) * iz;
                        p2.v[k] = bc * iz;
                    } else {
                        p1.v[k] = -0.5f * bc * iz;
                    }
                }
            }
        }
        store<V>(m1 + (size_t)idx * V, p1);
        if (kTwoMaps) store<V>(m2 + (size_t)idx * V, p2);
    }
    __syncthreads();

    // phase 2: window sums for one pixel and V channels, then that element's output
    for (int idx = tid; idx < kTileH * kTileW * CBV; idx += 256) {
        const int op = idx / CBV, cv = idx - op * CBV;
        const int oi = op / kTileW, oj = op - oi * kTileW;
        const int row = ti + oi, col = tj + oj;
        if (cv >= ncv || row >= H || col >= W) continue;
        float s1[V], s2[V];
#pragma unroll
        for (int k = 0; k < V; ++k) s1[k] = s2[k] = 0.f;
        for (int p = 0; p < a.ks; ++p)
            for (int q = 0; q < a.ks; ++q) {
                const float wt = a.taps.g[p] * a.taps.g[q];
                const int h = (((oi + p) * hw + oj + q) * CBV + cv) * V;
                const Pack<V> t = load<V>(m1 + h);
                if (OP == kBwdOne) {
                    const Pack<V> t2 = load<V>(m2 + h);
#pragma unroll
                    for (int k = 0; k < V; ++k) { s1[k] += wt * t.v[k]; s2[k] += wt * t2.v[k]; }
                } else {
#pragma unroll
                    for (int k = 0; k < V; ++k) {
                        if (OP == kDivide) s1[k] += wt * t.v[k] * t.v[k];
                        else s1[k] += wt * t.v[k];
                        if (OP == kFwdOne) s2[k] += wt * t.v[k] * t.v[k];
                    }
                }
            }
        const size_t e = (img + (size_t)row * W + col) * C + c0 + cv * V;
        const float z = norm_at(row, col);
        Pack<V> o;
        if (OP == kFwdOne || OP == kDivide) {
            // the element's own x (or x - mu) is still in LDS
            const Pack<V> ctr = load<V>(m1 + (((oi + r) * hw + oj + r) * CBV + cv) * V);
            Pack<V> m, rs;
#pragma unroll
            for (int k = 0; k < V; ++k) {
                if (OP == kFwdOne) {
                    m.v[k] = s1[k] / z;
                    rs.v[k] = 1.0f / sqrtf(fmaxf(s2[k] / z - m.v[k] * m.v[k], 0.f) + a.eps);
                    o.v[k] = (ctr.v[k] - m.v[k]) * rs.v[k];
                } else {
                    rs.v[k] = 1.0f / sqrtf(s1[k] / z + a.eps);
                    o.v[k] = ctr.v[k] * rs.v[k];
                }
            }
            if (OP == kFwdOne) store<V>(a.mu_out + e, m);
            store<V>(a.rstd_out + e, rs);
            store<V>(a.out + e, o);
        } else if (OP == kMean) {
#pragma unroll
            for (int k = 0; k < V; ++k) o.v[k] = s1[k] / z;
            store<V>(a.mu_out + e, o);
        } else if (OP == kBwdOne) {
            const Pack<V> xv = load<V>(a.x + e), dv = load<V>(a.dy + e), rs = load<V>(a.rstd_in + e);
#pragma unroll
            for (int k = 0; k < V; ++k) o.v[k] = dv.v[k] * rs.v[k] + s1[k] - xv.v[k] * s2[k];
            store<V>(a.out + e, o);
        } else if (OP == kBwdTwoA) {
            const Pack<V> xv = load<V>(a.x + e), dv = load<V>(a.dy + e), m = load<V>(a.mu_in + e),
                          rs = load<V>(a.rstd_in + e);
            Pack<V> f;
#pragma unroll
            for (int k = 0; k < V; ++k) {
                o.v[k] = dv.v[k] * rs.v[k] + 2.f * (xv.v[k] - m.v[k]) * s1[k];
                f.v[k] = o.v[k] / z;
            }
            store<V>(a.out + e, o);
            store<V>(a.field + e, f);
        } else {   // kBwdTwoB
            const Pack<V> dv = load<V>(a.out + e);
#pragma unroll
            for (int k = 0; k < V; ++k) o.v[k] = dv.v[k] - s1[k];
            store<V>(a.out + e, o);
        }
    }
}

bool make_taps(int ks, float sigma, Taps *t) {
    if (ks < 1 || ks > kMaxK || (ks & 1) == 0 || !(sigma > 0.f)) return false;
    const int r = (ks - 1) / 2;
    double s = 0.0, g[kMaxK];
    for (int p = -r; p <= r; ++p) {
        g[p + r] = exp(-(double)(p * p) / (2.0 * (double)sigma * (double)sigma));
        s += g[p + r];
    }
    for (int p = 0; p < kMaxK; ++p) t->g[p] = p < ks ? (float)(g[p] / s) : 0.f;
    return true;
}

template <int OP, int V>
int launch_pass_v(Args a, int B, hipStream_t s, const char *where) {
    const int tiles_h = (a.H + kTileH - 1) / kTileH;
    a.tiles_w = (a.W + kTileW - 1) / kTileW;
    a.tiles_per_img = tiles_h * a.tiles_w;
    const int maps = OP == kBwdOne ? 2 : 1;
    const size_t per_channel = (size_t)(kTileH + a.ks - 1) * (kTileW + a.ks - 1) * maps * sizeof(float);
    // whole 128-byte lines of a pixel where LDS allows; never fewer than V channels (at most 10.6 KB then)
    a.CB = a.C < 32 ? a.C : 32;
    while (a.CB > V && a.CB * per_channel > (size_t)kLdsTarget) a.CB = (a.CB / 2 + V - 1) / V * V;
    a.nchunk = (a.C + a.CB - 1) / a.CB;
    const long long nblk = (long long)B * a.tiles_per_img * a.nchunk;
    if (nblk > 0x7fffffffLL) return LC_EUNSUPPORTED;
    const size_t lds = a.CB * per_channel;
    auto kern = lcn_channel_kernel<OP, V>;
    if (int rc = allow_dynamic_lds((const void *)kern, lds, where)) return rc;
    hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(256), lds, s, a);
    LC_HIP_LAUNCH_CHECK(where);
    return LC_OK;
}

template <int OP>
int launch_pass(const Args &a, int B, hipStream_t s, const char *where) {
    return a.C % 4 == 0 ? launch_pass_v<OP, 4>(a, B, s, where) : launch_pass_v<OP, 1>(a, B, s, where);
}

}  // namespace

size_t lcn_variant_scratch_bytes(int B, int H, int W, int C, unsigned flags) {
    if (!(flags & LCN_TWO_STAGE)) return 0;
    return (size_t)B * H * W * ((flags & LCN_PER_CHANNEL) ? C : 1) * sizeof(float);
}

int launch_lcn_variant_fwd(const float *x, float *y, float *mu, float *rstd, int B, int H, int W, int C, int ks,
                           float sigma, float eps, unsigned flags, hipStream_t s) {
    const bool pc = flags & LCN_PER_CHANNEL, zp = flags & LCN_ZERO_PAD, two = flags & LCN_TWO_STAGE;
    if (!pc) {
        if (!two) return launch_lcn(0, x, nullptr, y, mu, rstd, B, H, W, C, ks, sigma, eps, s, zp);
        if (int rc = launch_lcn(2, x, nullptr, y, mu, rstd, B, H, W, C, ks, sigma, eps, s, zp)) return rc;
        return launch_lcn(3, x, nullptr, y, mu, rstd, B, H, W, C, ks, sigma, eps, s, zp);
    }
    Args a{};
    if (!make_taps(ks, sigma, &a.taps)) return LC_EINVAL;
    a.x = x; a.out = y; a.mu_out = mu; a.rstd_out = rstd; a.mu_in = mu;
    a.H = H; a.W = W; a.C = C; a.ks = ks; a.zpad = zp; a.eps = eps;
    if (!two) return launch_pass<kFwdOne>(a, B, s, "lcn_variant_fwd");
    if (int rc = launch_pass<kMean>(a, B, s, "lcn_variant_fwd (mean)")) return rc;
    return launch_pass<kDivide>(a, B, s, "lcn_variant_fwd (divide)");
}

int launch_lcn_variant_bwd(const float *x, const float *mu, const float *rstd, const float *dy, float *dx, int B, int H,
                           int W, int C, int ks, float sigma, unsigned flags, void *ws, size_t ws_bytes, hipStream_t s) {
    const bool pc = flags & LCN_PER_CHANNEL, zp = flags & LCN_ZERO_PAD, two = flags & LCN_TWO_STAGE;
    if (two && (ws == nullptr || ws_bytes < lcn_variant_scratch_bytes(B, H, W, C, flags))) return LC_EWORKSPACE;
    float *mu_ = const_cast<float *>(mu), *rstd_ = const_cast<float *>(rstd);   // read only in these modes
    if (!pc) {
        if (!two) return launch_lcn(1, x, dy, dx, mu_, rstd_, B, H, W, C, ks, sigma, 0.f, s, zp);
        if (int rc = launch_lcn(4, x, dy, dx, mu_, rstd_, B, H, W, C, ks, sigma, 0.f, s, zp, (float *)ws)) return rc;
        return launch_lcn(5, x, dy, dx, mu_, rstd_, B, H, W, C, ks, sigma, 0.f, s, zp, (float *)ws);
    }
    Args a{};
    if (!make_taps(ks, sigma, &a.taps)) return LC_EINVAL;
    a.x = x; a.dy = dy; a.mu_in = mu; a.rstd_in = rstd; a.out = dx; a.field = (float *)ws;
    a.H = H; a.W = W; a.C = C; a.ks = ks; a.zpad = zp;
    if (!two) return launch_pass<kBwdOne>(a, B, s, "lcn_variant_bwd");
    if (int rc = launch_pass<kBwdTwoA>(a, B, s, "lcn_variant_bwd (dv)")) return rc;
    return launch_pass<kBwdTwoB>(a, B, s, "lcn_variant_bwd (mean)");
}

}  // namespace lc

// ---------------------------------------------------------------------------------------------
// lcn_variant_bwd_static: lcn_variant_bwd for callers that cannot allocate.  The scratch field of the two-stage
// gradient (one float per statistic) lives in a file-scope device array instead of a caller's workspace.  Every GPU
// the library runs on holds its own copy of the array at its own address until the process ends; the address is
// looked up once per device, on the first call there, and only that pointer (never the array's name, which in host
// code is a stand-in and no device address) is handed to the kernels.  Nothing in the array has to start at zero:
// the first pass writes every element the second pass reads.
namespace lc {
namespace {

constexpr size_t kStaticScratchBytes = (size_t)LCN_STATIC_SCRATCH_BYTES;
__device__ __align__(256) unsigned char lcn_static_scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// the calling thread's current device's copy of the array; LC_OK or LC_EHIP
int static_scratch(void **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_hip_error(e, "lcn_variant_bwd_static: hipGetDevice"); return LC_EHIP; }
    if (dev < 0 || dev >= kMaxDevices) { set_error_text("lcn_variant_bwd_static: device index out of range"); return LC_EHIP; }
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(lcn_static_scratch));
        if (e != hipSuccess || !p) { set_hip_error(e, "lcn_variant_bwd_static: hipGetSymbolAddress"); return LC_EHIP; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LC_OK;
}

}  // namespace
}  // namespace lc

extern "C" int lcn_variant_bwd_static(const float *x, const float *mu, const float *rstd, const float *dy, float *dx,
                                      int32_t B, int32_t H, int32_t W, int32_t C, int32_t ksize, float gauss_sigma,
                                      uint32_t flags, void *hip_stream) {
    using namespace lc;
    if (int rc = check_lcn_variant_bwd_args(x, mu, rstd, dy, dx, B, H, W, C, ksize, gauss_sigma, flags)) return rc;
    const size_t need = lcn_variant_scratch_bytes(B, H, W, C, flags);
    if (need > kStaticScratchBytes) {
        set_error_text("lcn_variant_bwd_static: the two-stage gradient of this map needs more scratch than the "
                       "library's static array holds (LCN_STATIC_SCRATCH_BYTES); use lcn_variant_bwd with a workspace");
        return LC_EWORKSPACE;
    }
    void *scratch = nullptr;
    if (need > 0)
        if (int rc = static_scratch(&scratch)) return rc;
    return launch_lcn_variant_bwd(x, mu, rstd, dy, dx, B, H, W, C, ksize, gauss_sigma, flags, scratch, need,
                                  (hipStream_t)hip_stream);
}

