// Variants of the local contrast normalisation applied after each layer (Sec. 3.1 names LCN without defining it):
// statistics per channel instead of pooled over the channels, zero-padded instead of renormalised borders, and
// the two-stage form (subtract the local mean, then divide by the local root mean square of the result).
//
// One kernel template covers every pass.  A "statistic" is a pixel (pooled: it owns the pixel's CR = C channels)
// or a pixel and channel (per channel: CR = 1).  A workgroup takes a 16x16 pixel tile and up to SC statistics per
// pixel; it reduces a per-statistic quantity over the tile and its halo into LDS, forms the Gaussian window sums,
// and finishes with the elementwise pass over the elements its statistics own.  Bandwidth-bound: the tile is
// read once or twice, the halo ring comes from L2.
#include "lc_common.hpp"

namespace lc {
namespace {

constexpr int kTile = 16;
constexpr int kMaxK = 15;
constexpr int kMaxStatsPerBlock = 8;

struct Taps { float g[kMaxK]; };

enum : int {
    kFwdOne,    // x -> mu, rstd, y (one stage)
    kMean,      // x -> mu
    kDivide,    // x, mu -> rstd, y = (x - mu) rstd with the window mean of the neighbours' own (x - mu)^2
    kBwdOne,    // one-stage gradient
    kBwdTwoA,   // two-stage gradient up to dv (written to dx) and the per-statistic sums of dv / normaliser
    kBwdTwoB    // dx = dv - window sum of those sums
};

struct Args {
    const float *x, *dy, *mu_in, *rstd_in;
    float *out, *mu_out, *rstd_out, *field;
    int H, W, CS, CR, SC, ks, zpad, tiles_w, tiles_per_img, nchunk;
    float eps;
    Taps taps;
};

__device__ __forceinline__ float taps_inside(const Taps &t, int p, int n, int r) {
    float z = 0.f;
    for (int d = -r; d <= r; ++d)
        if (p + d >= 0 && p + d < n) z += t.g[d + r];
    return z;
}

template <int OP>
__global__ __launch_bounds__(256) void lcn_variant_kernel(Args a) {
    extern __shared__ float lds[];
    constexpr bool kTwoMaps = OP == kFwdOne || OP == kBwdOne;
    const int r = (a.ks - 1) / 2, halo = kTile + 2 * r, SC = a.SC, CR = a.CR, CS = a.CS, H = a.H, W = a.W;
    float *m1 = lds, *m2 = lds + halo * halo * SC;
    const int tid = threadIdx.x;
    int blk = blockIdx.x;
    const int chunk = blk % a.nchunk;
    blk /= a.nchunk;
    const int b = blk / a.tiles_per_img, tile = blk - b * a.tiles_per_img;
    const int ti = (tile / a.tiles_w) * kTile, tj = (tile % a.tiles_w) * kTile;
    const int sc0 = chunk * SC, nsc = min(SC, CS - sc0);
    const size_t img = (size_t)b * H * W;
    const float zc = (float)CR;

    // the normaliser of the statistic centred on (row, col)
    auto norm_at = [&](int row, int col) {
        return (a.zpad ? 1.f : taps_inside(a.taps, row, H, r) * taps_inside(a.taps, col, W, r)) * zc;
    };

    // phase 1: one quantity (or two) per statistic of the tile and its halo; zeros outside the image
    for (int idx = tid; idx < halo * halo * SC; idx += 256) {
        const int hp = idx / SC, sc = idx - hp * SC;
        const int hi = hp / halo, hj = hp - hi * halo;
        const int row = ti - r + hi, col = tj - r + hj;
        float p1 = 0.f, p2 = 0.f;
        if (sc < nsc && row >= 0 && row < H && col >= 0 && col < W) {
            const size_t st = (img + (size_t)row * W + col) * CS + sc0 + sc;
            const size_t e0 = st * CR;
            if (OP == kBwdTwoB) {
                p1 = a.field[st];
            } else {
                float m = 0.f, rs = 0.f;
                if (OP == kDivide || OP == kBwdOne || OP == kBwdTwoA) m = a.mu_in[st];
                if (OP == kBwdOne || OP == kBwdTwoA) rs = a.rstd_in[st];
                float s1 = 0.f, s2 = 0.f;
                auto take = [&](float xv, float dv) {
                    if (OP == kFwdOne) { s1 += xv; s2 += xv * xv; }
                    if (OP == kMean) s1 += xv;
                    if (OP == kDivide) s1 += (xv - m) * (xv - m);
                    if (OP == kBwdOne) { s1 += dv; s2 += dv * (xv - m); }
                    if (OP == kBwdTwoA) s2 += dv * (xv - m);
                };
                constexpr bool kNeedDy = OP == kBwdOne || OP == kBwdTwoA;
                if ((CR & 3) == 0) {
                    for (int c = 0; c < CR; c += 4) {
                        const float4 xv = *(const float4 *)(a.x + e0 + c);
                        float4 dv = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (kNeedDy) dv = *(const float4 *)(a.dy + e0 + c);
                        take(xv.x, dv.x); take(xv.y, dv.y); take(xv.z, dv.z); take(xv.w, dv.w);
                    }
                } else {
                    for (int c = 0; c < CR; ++c) take(a.x[e0 + c], kNeedDy ? a.dy[e0 + c] : 0.f);
                }
                if (OP == kFwdOne) { p1 = s1; p2 = s2; }
                if (OP == kMean || OP == kDivide) p1 = s1;
                if (OP == kBwdOne) {
                    // gradients of this statistic's mean and second moment, already divided by its normaliser
                    const float z = norm_at(row, col), bc = rs * rs * rs * s2;
                    p1 = (bc * m - rs * s1) / z;
                    p2 = bc / z;
                }
                if (OP == kBwdTwoA) p1 = -0.5f * rs * rs * rs * s2 / norm_at(row, col);
            }
        }
        m1[idx] = p1;
        if (kTwoMaps) m2[idx] = p2;
    }
    __syncthreads();

    // phase 2: window sums for the tile's statistics, then the elementwise pass over what each one owns
    for (int idx = tid; idx < kTile * kTile * SC; idx += 256) {
        const int op = idx / SC, sc = idx - op * SC;
        const int oi = op / kTile, oj = op - oi * kTile;
        const int row = ti + oi, col = tj + oj;
        if (sc >= nsc || row >= H || col >= W) continue;
        float s1 = 0.f, s2 = 0.f;
        for (int p = 0; p < a.ks; ++p)
            for (int q = 0; q < a.ks; ++q) {
                const float wt = a.taps.g[p] * a.taps.g[q];
                const int h = ((oi + p) * halo + oj + q) * SC + sc;
                s1 += wt * m1[h];
                if (kTwoMaps) s2 += wt * m2[h];
            }
        const size_t st = (img + (size_t)row * W + col) * CS + sc0 + sc;
        const size_t e0 = st * CR;
        float u = 0.f, v = 0.f;   // the two per-statistic factors of the elementwise pass
        if (OP == kFwdOne) {
            const float z = norm_at(row, col);
            u = s1 / z;
            v = 1.0f / sqrtf(fmaxf(s2 / z - u * u, 0.f) + a.eps);
            a.mu_out[st] = u;
            a.rstd_out[st] = v;
        }
        if (OP == kMean) {
            a.mu_out[st] = s1 / norm_at(row, col);
            continue;
        }
        if (OP == kDivide) {
            u = a.mu_in[st];
            v = 1.0f / sqrtf(s1 / norm_at(row, col) + a.eps);
            a.rstd_out[st] = v;
        }
        if (OP == kBwdOne) { u = s1; v = s2; }
        if (OP == kBwdTwoA || OP == kBwdTwoB) u = s1;
        float rs = 0.f, m = 0.f, acc = 0.f;
        if (OP == kBwdOne || OP == kBwdTwoA) rs = a.rstd_in[st];
        if (OP == kBwdTwoA) m = a.mu_in[st];
        auto each = [&](float xv, float dv, float ov) -> float {
            if (OP == kFwdOne || OP == kDivide) return (xv - u) * v;
            if (OP == kBwdOne) return dv * rs + u - xv * v;
            if (OP == kBwdTwoA) {
                const float g = dv * rs + 2.f * (xv - m) * u;
                acc += g;
                return g;
            }
            return ov - u;   // kBwdTwoB
        };
        constexpr bool kNeedX = OP != kBwdTwoB, kNeedDy = OP == kBwdOne || OP == kBwdTwoA, kNeedOut = OP == kBwdTwoB;
        if ((CR & 3) == 0) {
            const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int c = 0; c < CR; c += 4) {
                const float4 xv = kNeedX ? *(const float4 *)(a.x + e0 + c) : zero;
                const float4 dv = kNeedDy ? *(const float4 *)(a.dy + e0 + c) : zero;
                const float4 ov = kNeedOut ? *(const float4 *)(a.out + e0 + c) : zero;
                *(float4 *)(a.out + e0 + c) =
                    make_float4(each(xv.x, dv.x, ov.x), each(xv.y, dv.y, ov.y), each(xv.z, dv.z, ov.z), each(xv.w, dv.w, ov.w));
            }
        } else {
            for (int c = 0; c < CR; ++c)
                a.out[e0 + c] = each(kNeedX ? a.x[e0 + c] : 0.f, kNeedDy ? a.dy[e0 + c] : 0.f, kNeedOut ? a.out[e0 + c] : 0.f);
        }
        if (OP == kBwdTwoA) a.field[st] = acc / norm_at(row, col);
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

template <int OP>
int launch_pass(Args a, int B, hipStream_t s, const char *where) {
    const int tiles_h = (a.H + kTile - 1) / kTile;
    a.tiles_w = (a.W + kTile - 1) / kTile;
    a.tiles_per_img = tiles_h * a.tiles_w;
    a.SC = a.CS < kMaxStatsPerBlock ? a.CS : kMaxStatsPerBlock;
    a.nchunk = (a.CS + a.SC - 1) / a.SC;
    const long long nblk = (long long)B * a.tiles_per_img * a.nchunk;
    if (nblk > 0x7fffffffLL) return LC_EUNSUPPORTED;
    const int halo = kTile + a.ks - 1;
    const bool two_maps = OP == kFwdOne || OP == kBwdOne;
    const size_t lds = (size_t)halo * halo * a.SC * sizeof(float) * (two_maps ? 2 : 1);   // at most 57.6 KB
    auto kern = lcn_variant_kernel<OP>;
    if (int rc = allow_dynamic_lds((const void *)kern, lds, where)) return rc;
    hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(256), lds, s, a);
    LC_HIP_LAUNCH_CHECK(where);
    return LC_OK;
}

}  // namespace

size_t lcn_variant_scratch_bytes(int B, int H, int W, int C, unsigned flags) {
    if (!(flags & LCN_TWO_STAGE)) return 0;
    return (size_t)B * H * W * ((flags & LCN_PER_CHANNEL) ? C : 1) * sizeof(float);
}

int launch_lcn_variant_fwd(const float *x, float *y, float *mu, float *rstd, int B, int H, int W, int C, int ks,
                           float sigma, float eps, unsigned flags, hipStream_t s) {
    const bool pc = flags & LCN_PER_CHANNEL, zp = flags & LCN_ZERO_PAD, two = flags & LCN_TWO_STAGE;
    // pooled one-stage statistics: the wavefront-reduction kernels of the default form
    if (!pc && !two) return launch_lcn(0, x, nullptr, y, mu, rstd, B, H, W, C, ks, sigma, eps, s, zp);
    Args a{};
    if (!make_taps(ks, sigma, &a.taps)) return LC_EINVAL;
    a.x = x; a.out = y; a.mu_out = mu; a.rstd_out = rstd; a.mu_in = mu;
    a.H = H; a.W = W; a.CS = pc ? C : 1; a.CR = pc ? 1 : C; a.ks = ks; a.zpad = zp; a.eps = eps;
    if (!two) return launch_pass<kFwdOne>(a, B, s, "lcn_variant_fwd");
    if (int rc = launch_pass<kMean>(a, B, s, "lcn_variant_fwd (mean)")) return rc;
    return launch_pass<kDivide>(a, B, s, "lcn_variant_fwd (divide)");
}

int launch_lcn_variant_bwd(const float *x, const float *mu, const float *rstd, const float *dy, float *dx, int B, int H,
                           int W, int C, int ks, float sigma, unsigned flags, void *ws, size_t ws_bytes, hipStream_t s) {
    const bool pc = flags & LCN_PER_CHANNEL, zp = flags & LCN_ZERO_PAD, two = flags & LCN_TWO_STAGE;
    if (!pc && !two)
        return launch_lcn(1, x, dy, dx, const_cast<float *>(mu), const_cast<float *>(rstd), B, H, W, C, ks, sigma, 0.f, s,
                          zp);
    Args a{};
    if (!make_taps(ks, sigma, &a.taps)) return LC_EINVAL;
    a.x = x; a.dy = dy; a.mu_in = mu; a.rstd_in = rstd; a.out = dx;
    a.H = H; a.W = W; a.CS = pc ? C : 1; a.CR = pc ? 1 : C; a.ks = ks; a.zpad = zp;
    if (!two) return launch_pass<kBwdOne>(a, B, s, "lcn_variant_bwd");
    if (ws == nullptr || ws_bytes < lcn_variant_scratch_bytes(B, H, W, C, flags)) return LC_EWORKSPACE;
    a.field = (float *)ws;
    if (int rc = launch_pass<kBwdTwoA>(a, B, s, "lcn_variant_bwd (dv)")) return rc;
    return launch_pass<kBwdTwoB>(a, B, s, "lcn_variant_bwd (mean)");
}

}  // namespace lc
