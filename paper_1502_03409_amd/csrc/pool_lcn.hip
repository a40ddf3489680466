// L2 pooling and local contrast normalisation, forward and backward.  Bandwidth-bound stencils over
// [B][H][W][C] activations: every kernel reads its inputs once from HBM (neighbour re-reads are served
// by L1/L2) and writes its output once.
//
// Pooling is not part of the paper's network (Sec. 3.1 leaves it out); LCN is applied after each layer
// (Sec. 3.1) and is taken here as Gaussian-windowed local standardisation with statistics pooled over
// the channels: the channel sums are wavefront reductions, the window sums a small LDS stencil.
#include <algorithm>

#include "lc_common.hpp"

namespace lc {

// threads per workgroup of the band kernels: a band of whole image rows lives in their registers (512 threads with
// bands half as long measured the same)
constexpr int kBandThreads = 1024;

// ------------------------------------------------------------------ L2 pooling
template <int VEC>
__global__ __launch_bounds__(256) void l2pool_fwd_kernel(const float *__restrict__ x, float *__restrict__ y, int B,
                                                         int H, int W, int C, int Ho, int Wo, int ks, int st,
                                                         float eps, long long total) {
    const int CV = C / VEC;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
        const int cv = (int)(e % CV);
        long long t = e / CV;
        const int j = (int)(t % Wo);
        t /= Wo;
        const int i = (int)(t % Ho), b = (int)(t / Ho);
        const float *xp = x + (((size_t)b * H + (size_t)i * st) * W + (size_t)j * st) * C + cv * VEC;
        float s[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) s[v] = 0.f;
        for (int p = 0; p < ks; ++p)
            for (int q = 0; q < ks; ++q) {
                const float *src = xp + ((size_t)p * W + q) * C;
                if (VEC == 4) {
                    const float4 t4 = *(const float4 *)src;
                    s[0] += t4.x * t4.x; s[1 % VEC] += t4.y * t4.y; s[2 % VEC] += t4.z * t4.z; s[3 % VEC] += t4.w * t4.w;
                } else {
                    s[0] += src[0] * src[0];
                }
            }
        float *dst = y + (size_t)e * VEC;
        if (VEC == 4)
            *(float4 *)dst = make_float4(sqrtf(eps + s[0]), sqrtf(eps + s[1 % VEC]), sqrtf(eps + s[2 % VEC]),
                                         sqrtf(eps + s[3 % VEC]));
        else
            dst[0] = sqrtf(eps + s[0]);
    }
}

template <int VEC>
__global__ __launch_bounds__(256) void l2pool_bwd_kernel(const float *__restrict__ x, const float *__restrict__ y,
                                                         const float *__restrict__ dy, float *__restrict__ dx, int B,
                                                         int H, int W, int C, int Ho, int Wo, int ks, int st,
                                                         long long total) {
    const int CV = C / VEC;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
        const int cv = (int)(e % CV);
        long long t = e / CV;
        const int col = (int)(t % W);
        t /= W;
        const int row = (int)(t % H), b = (int)(t / H);
        // windows (i,j) with i*st <= row < i*st+ks
        const int i_hi = min(row / st, Ho - 1), j_hi = min(col / st, Wo - 1);
        const int i_lo = max(0, (row - ks + st) / st), j_lo = max(0, (col - ks + st) / st);
        float s[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) s[v] = 0.f;
        for (int i = i_lo; i <= i_hi; ++i)
            for (int j = j_lo; j <= j_hi; ++j) {
                const size_t o = (((size_t)b * Ho + i) * Wo + j) * C + cv * VEC;
                if (VEC == 4) {
                    const float4 g4 = *(const float4 *)(dy + o), y4 = *(const float4 *)(y + o);
                    s[0] += g4.x / y4.x; s[1 % VEC] += g4.y / y4.y; s[2 % VEC] += g4.z / y4.z; s[3 % VEC] += g4.w / y4.w;
                } else {
                    s[0] += dy[o] / y[o];
                }
            }
        const size_t xo = (size_t)e * VEC;
        if (VEC == 4) {
            const float4 x4 = *(const float4 *)(x + xo);
            *(float4 *)(dx + xo) = make_float4(x4.x * s[0], x4.y * s[1 % VEC], x4.z * s[2 % VEC], x4.w * s[3 % VEC]);
        } else {
            dx[xo] = x[xo] * s[0];
        }
    }
}

// Stride-1 windows, C % 4 == 0: a thread owns OW consecutive output columns of one (image, row, channel
// quad) and keeps the per-column partial sums in registers, so every input is loaded ks times (once
// per output row it belongs to) instead of ks*ks times.
constexpr int kPoolOW = 4;
constexpr int kPoolMaxK = 5;

__global__ __launch_bounds__(256) void l2pool_fwd_rows_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                              int H, int W, int C, int Ho, int Wo, int ks, float eps,
                                                              int groups) {
    // grid: x over (output row, column group, channel quad) of one image, y = image
    const int CV = C >> 2;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= Ho * groups * CV) return;
    const int t = e / CV, cv = e - t * CV;
    const int i = t / groups, jg = t - i * groups;
    const int b = blockIdx.y;
    const int j0 = jg * kPoolOW;
    const int ncol = min(kPoolOW, Wo - j0) + ks - 1;          // input columns this thread needs
    f32x4 col[kPoolOW + kPoolMaxK - 1];
#pragma unroll
    for (int c = 0; c < kPoolOW + kPoolMaxK - 1; ++c) col[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const float *xp = x + (((size_t)b * H + i) * W + j0) * C + cv * 4;
    for (int p = 0; p < ks; ++p) {
#pragma unroll
        for (int c = 0; c < kPoolOW + kPoolMaxK - 1; ++c) {
            if (c < ncol) {
                const f32x4 v = *(const f32x4 *)(xp + ((size_t)p * W + c) * C);
                col[c] += v * v;
            }
        }
    }
    float *yp = y + (((size_t)b * Ho + i) * Wo + j0) * C + cv * 4;
#pragma unroll
    for (int o = 0; o < kPoolOW; ++o) {
        if (j0 + o < Wo) {
            f32x4 sacc = (f32x4){eps, eps, eps, eps};
#pragma unroll
            for (int q = 0; q < kPoolMaxK; ++q)
                if (q < ks) sacc += col[o + q];
            *(f32x4 *)(yp + (size_t)o * C) =
                (f32x4){sqrtf(sacc[0]), sqrtf(sacc[1]), sqrtf(sacc[2]), sqrtf(sacc[3])};
        }
    }
}

// Backward, same shapes: a thread owns OW consecutive input columns of one (image, row, channel quad); the
// per-column sums of dy/y over the output rows that cover this input row are kept in registers.
__global__ __launch_bounds__(256) void l2pool_bwd_rows_kernel(const float *__restrict__ x, const float *__restrict__ y,
                                                              const float *__restrict__ dy, float *__restrict__ dx,
                                                              int H, int W, int C, int Ho, int Wo, int ks, int groups) {
    // grid: x over (input row, column group, channel quad) of one image, y = image
    const int CV = C >> 2;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= H * groups * CV) return;
    const int t = e / CV, cv = e - t * CV;
    const int row = t / groups, jg = t - row * groups;
    const int b = blockIdx.y;
    const int c0 = jg * kPoolOW;                               // first input column
    const int i_lo = max(0, row - ks + 1), i_hi = min(row, Ho - 1);
    // output columns jo in [c0-ks+1, c0+OW-1] may cover this thread's inputs
    f32x4 col[kPoolOW + kPoolMaxK - 1];
#pragma unroll
    for (int c = 0; c < kPoolOW + kPoolMaxK - 1; ++c) col[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int i = i_lo; i <= i_hi; ++i) {
        const size_t rb = (((size_t)b * Ho + i) * Wo) * C + cv * 4;
#pragma unroll
        for (int c = 0; c < kPoolOW + kPoolMaxK - 1; ++c) {
            const int jo = c0 - (ks - 1) + c;
            if (c < kPoolOW + ks - 1 && jo >= 0 && jo < Wo) {
                const f32x4 g = *(const f32x4 *)(dy + rb + (size_t)jo * C), yy = *(const f32x4 *)(y + rb + (size_t)jo * C);
                col[c] += g / yy;
            }
        }
    }
    const size_t xo = (((size_t)b * H + row) * W + c0) * C + cv * 4;
#pragma unroll
    for (int o = 0; o < kPoolOW; ++o) {
        if (c0 + o < W) {
            // input column c0+o is covered by output columns jo = c0+o-ks+1 .. c0+o, i.e. col[o .. o+ks-1]
            f32x4 sacc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < kPoolMaxK; ++q)
                if (q < ks) sacc += col[o + q];
            *(f32x4 *)(dx + xo + (size_t)o * C) = *(const f32x4 *)(x + xo + (size_t)o * C) * sacc;
        }
    }
}

// Tiled variant for stride-1 windows and C % 4 == 0: a workgroup stages the (TH+ks-1) x (TW+ks-1) patch its
// TH x TW tile needs in LDS once (forward: x^2; backward: dy/y), so every input leaves L2 about once instead
// of once per window row, and the window sums come out of LDS.
constexpr int kPoolTH = 8, kPoolTW = 16;

// MODE 0: y = sqrt(eps + window sum of x^2) on a tile of outputs.
// MODE 1: dx = x * (window sum of dy/y) on a tile of inputs; the patch holds dy/y at outputs
//         (row-ks+1 .. row, col-ks+1 .. col), zero where no such output exists.
// MODE 2: the same with dy/y handed in as one array (in `dy`; `y` is not read).
template <int MODE>
__global__ __launch_bounds__(256) void l2pool_tile_kernel(const float *__restrict__ x, const float *__restrict__ y,
                                                          const float *__restrict__ dy, float *__restrict__ out,
                                                          int H, int W, int C, int Ho, int Wo, int ks, float eps,
                                                          int tiles_w, int tiles_per_img) {
    extern __shared__ __attribute__((aligned(16))) float patch[];   // [(TH+ks-1)*(TW+ks-1)][C]
    const int tid = threadIdx.x, CV = C >> 2;
    // each XCD walks a contiguous range of tiles: the tiles of one image, whose halos overlap, share an L2
    const int blk = remap_xcd(blockIdx.x, gridDim.x);
    const int b = blk / tiles_per_img, tile = blk - b * tiles_per_img;
    const int ti = (tile / tiles_w) * kPoolTH, tj = (tile % tiles_w) * kPoolTW;
    const int PH = kPoolTH + ks - 1, PW = kPoolTW + ks - 1;
    // patch origin in the source grid: forward reads inputs (ti.., tj..); backward reads outputs (ti-ks+1.., tj-ks+1..)
    const int oi0 = MODE == 0 ? ti : ti - (ks - 1), oj0 = MODE == 0 ? tj : tj - (ks - 1);
    const int SH = MODE == 0 ? H : Ho, SW = MODE == 0 ? W : Wo;
    const size_t sbase = (size_t)b * SH * SW;
    // eight loads in flight per thread before the first goes to LDS
    const int npatch = PH * PW * CV;
    for (int e0 = tid; e0 < npatch; e0 += 256 * 8) {
        f32x4 v[8], v2[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int e = e0 + 256 * q;
            const int cv = e % CV, pp = e / CV;
            const int pi = pp / PW, pj = pp - pi * PW;
            const int r = oi0 + pi, c = oj0 + pj;
            v[q] = (f32x4){0.f, 0.f, 0.f, 0.f};
            v2[q] = (f32x4){1.f, 1.f, 1.f, 1.f};
            if (e < npatch && r >= 0 && r < SH && c >= 0 && c < SW) {
                const size_t o = (sbase + (size_t)r * SW + c) * C + cv * 4;
                if (MODE == 0) {
                    v[q] = *(const f32x4 *)(x + o);
                } else {
                    v[q] = *(const f32x4 *)(dy + o);
                    if (MODE == 1) v2[q] = *(const f32x4 *)(y + o);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int e = e0 + 256 * q;
            if (e < npatch) *(f32x4 *)(patch + (size_t)e * 4) = MODE == 0 ? v[q] * v[q] : MODE == 1 ? v[q] / v2[q] : v[q];
        }
    }
    __syncthreads();
    // a thread owns 4 consecutive columns of one tile row and channel quad
    const int OH = MODE == 0 ? Ho : H, OWid = MODE == 0 ? Wo : W;
    for (int e = tid; e < kPoolTH * (kPoolTW / 4) * CV; e += 256) {
        const int cv = e % CV, t = e / CV;
        const int cg = t % (kPoolTW / 4), tr = t / (kPoolTW / 4);
        const int row = ti + tr, col0 = tj + cg * 4;
        if (row >= OH || col0 >= OWid) continue;
        f32x4 col[4 + kPoolMaxK - 1];
#pragma unroll
        for (int c = 0; c < 4 + kPoolMaxK - 1; ++c) col[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < ks; ++p) {
            const float *prow = patch + ((size_t)(tr + p) * PW + cg * 4) * C + cv * 4;
#pragma unroll
            for (int c = 0; c < 4 + kPoolMaxK - 1; ++c)
                if (c < 4 + ks - 1) col[c] += *(const f32x4 *)(prow + (size_t)c * C);
        }
        const size_t o = (((size_t)b * OH + row) * OWid + col0) * C + cv * 4;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (col0 + q >= OWid) continue;
            f32x4 sacc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < kPoolMaxK; ++k)
                if (k < ks) sacc += col[q + k];
            if (MODE == 0) {
                *(f32x4 *)(out + o + (size_t)q * C) =
                    (f32x4){sqrtf(eps + sacc[0]), sqrtf(eps + sacc[1]), sqrtf(eps + sacc[2]), sqrtf(eps + sacc[3])};
            } else {
                *(f32x4 *)(out + o + (size_t)q * C) = *(const f32x4 *)(x + o + (size_t)q * C) * sacc;
            }
        }
    }
}

// Forward pooling as a stream, stride 1 and a KS x KS window: a thread owns one output column and channel quad
// and walks down RS output rows.  Each input row it meets gives one horizontal sum of squares (KS loads whose
// neighbours in the wave read the same lines); the last KS-1 of them stay in registers, so an output costs one new
// row of loads.  No LDS and no barriers: every wave reads and writes all the time, and the loads of RU rows are in
// flight together.  Segments of RS rows re-read KS-1 input rows of the segment above.
template <int KS, int RU>
__global__ __launch_bounds__(256) void l2pool_fwd_stream_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                int H, int W, int CV, int Ho, int Wo, int RS,
                                                                int nseg, float eps, long long total) {
    const long long e = (long long)remap_xcd(blockIdx.x, gridDim.x) * 256 + threadIdx.x;
    if (e >= total) return;
    const int per_row = Wo * CV;
    const int cj = (int)(e % per_row);
    const long long t = e / per_row;
    const int sg = (int)(t % nseg), b = (int)(t / nseg);
    const int ro0 = sg * RS, ro1 = min(ro0 + RS, Ho);
    const size_t xrow = (size_t)W * CV, yrow = (size_t)Wo * CV;     // row strides in float4
    const f32x4 *xp = (const f32x4 *)x + (size_t)b * H * xrow + cj;  // column j, quad cv: offset j*CV + cv = cj
    f32x4 *yp = (f32x4 *)y + (size_t)b * Ho * yrow + cj;
    f32x4 ring[KS - 1];
#pragma unroll
    for (int d = 0; d < KS - 1; ++d) {
        const f32x4 *p = xp + (size_t)min(ro0 + d, H - 1) * xrow;
        f32x4 h = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int dj = 0; dj < KS; ++dj) { const f32x4 v = p[dj * CV]; h += v * v; }
        ring[d] = h;
    }
    for (int ro = ro0; ro < ro1; ro += RU) {
        f32x4 v[RU][KS];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            // rows past the segment are read from the last input row and never stored
            const f32x4 *p = xp + (size_t)min(ro + u + KS - 1, H - 1) * xrow;
#pragma unroll
            for (int dj = 0; dj < KS; ++dj) v[u][dj] = p[dj * CV];
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            f32x4 h = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int dj = 0; dj < KS; ++dj) h += v[u][dj] * v[u][dj];
            f32x4 sacc = h;
#pragma unroll
            for (int d = 0; d < KS - 1; ++d) sacc += ring[d];
            if (ro + u < ro1)
                yp[(size_t)(ro + u) * yrow] = (f32x4){sqrtf(eps + sacc[0]), sqrtf(eps + sacc[1]),
                                                      sqrtf(eps + sacc[2]), sqrtf(eps + sacc[3])};
#pragma unroll
            for (int d = 0; d + 1 < KS - 1; ++d) ring[d] = ring[d + 1];
            ring[KS - 2] = h;
        }
    }
}

// ------------------------------------------------------------------------ LCN
constexpr int kLcnTile = 16;   // output tile edge
constexpr int kLcnMaxK = 15;   // largest window
constexpr int kLcnHalo = kLcnTile + kLcnMaxK - 1;

struct GaussTaps { float g[kLcnMaxK]; };

__device__ __forceinline__ float group_sum(float v, int lpp) {
    for (int o = lpp >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// sum of the taps that stay inside [0,n) around position p (the normaliser of a window truncated at the border;
// with zero padding, zpad, the taps keep their full-window normalisation instead)
__device__ __forceinline__ float tap_norm(const GaussTaps &t, int p, int n, int r) {
    float z = 0.f;
    for (int d = -r; d <= r; ++d)
        if (p + d >= 0 && p + d < n) z += t.g[d + r];
    return z;
}

// Statistics pooled over the channels.  One-stage form: MODE 0 forward, MODE 1 backward (x, mu, rstd, dy -> dx).
// Two-stage form (subtract the window mean, divide by the root of the window mean of the neighbours' own squared
// differences) as two passes each way:
//   MODE 2  x -> mu;                          MODE 3  x, mu -> rstd, y = (x - mu) rstd;
//   MODE 4  x, mu, rstd, dy -> dv (into out) and field[p] = sum_c dv[p,c] / normaliser(p);
//   MODE 5  out = dv - window sum of field (in place).
template <int VEC, int MODE>
__global__ __launch_bounds__(256) void lcn_kernel(const float *__restrict__ x, const float *__restrict__ dy,
                                                  float *__restrict__ out, float *__restrict__ mu,
                                                  float *__restrict__ rstd, float *__restrict__ field, int H, int W,
                                                  int C, int ks, float eps, GaussTaps taps, int lpp, int tiles_w,
                                                  int tiles_per_img, int zpad) {
    constexpr bool kTwoMaps = MODE == 0 || MODE == 1;
    __shared__ float m1[kLcnHalo * kLcnHalo], m2[kTwoMaps ? kLcnHalo * kLcnHalo : 1];
    __shared__ float t1[kLcnTile * kLcnTile], t2[kLcnTile * kLcnTile];
    const int r = (ks - 1) / 2, halo = kLcnTile + 2 * r;
    const int tid = threadIdx.x;
    // each XCD walks a contiguous range of tiles: the tiles of one image, whose halos overlap, share an L2
    const int blk = remap_xcd(blockIdx.x, gridDim.x);
    const int b = blk / tiles_per_img, tile = blk - b * tiles_per_img;
    const int ti = (tile / tiles_w) * kLcnTile, tj = (tile % tiles_w) * kLcnTile;
    const int CV = C / VEC;
    const size_t img = (size_t)b * H * W;
    // window normalisers of the staged rows and columns, once per workgroup (a pixel's is their product times C)
    __shared__ float zr[kLcnHalo], zc[kLcnHalo];
    if (tid < halo) zr[tid] = zpad ? 1.f : tap_norm(taps, ti - r + tid, H, r);
    else if (tid >= 64 && tid < 64 + halo) zc[tid - 64] = zpad ? 1.f : tap_norm(taps, tj - r + tid - 64, W, r);
    if (MODE == 1 || MODE == 4) __syncthreads();   // the other modes first use them after phase 1's barrier
    auto norm_at = [&](int row, int col) { return zr[row - ti + r] * zc[col - tj + r] * (float)C; };

    // phase 1: per-pixel channel sums over the tile and its halo; lpp lanes share a pixel
    const int grp = tid / lpp, gl = tid % lpp, ngrp = 256 / lpp;
    for (int hp = grp; hp < halo * halo; hp += ngrp) {
        const int hi = hp / halo, hj = hp - hi * halo;
        const int row = ti - r + hi, col = tj - r + hj;
        float a = 0.f, c2 = 0.f;
        const bool in = row >= 0 && row < H && col >= 0 && col < W;
        // the pixel's own statistics are fetched with its values, not after the reduction
        float mp = 0.f, rsp = 0.f;
        if ((MODE == 1 || MODE == 3 || MODE == 4) && in) mp = mu[img + (size_t)row * W + col];
        if ((MODE == 1 || MODE == 4) && in) rsp = rstd[img + (size_t)row * W + col];
        if (MODE == 5) {
            if (in) a = field[img + (size_t)row * W + col];
        } else if (in) {
            const size_t pix = img + (size_t)row * W + col;
            const float *xp = x + pix * C;
            if (MODE == 0 || MODE == 2 || MODE == 3) {
                for (int cv = gl; cv < CV; cv += lpp) {
                    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (VEC == 4) v = *(const float4 *)(xp + cv * 4);
                    else v.x = xp[cv];
                    if (MODE == 3) {   // squared differences from the pixel's own mean (unused lanes of v stay out)
                        v.x -= mp;
                        if (VEC == 4) { v.y -= mp; v.z -= mp; v.w -= mp; }
                        a += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
                    } else {
                        a += (v.x + v.y) + (v.z + v.w);
                        c2 += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
                    }
                }
            } else {
                const float *gp = dy + pix * C;
                for (int cv = gl; cv < CV; cv += lpp) {
                    if (VEC == 4) {
                        const float4 v = *(const float4 *)(xp + cv * 4), d = *(const float4 *)(gp + cv * 4);
                        a += (d.x + d.y) + (d.z + d.w);
                        c2 += (d.x * (v.x - mp) + d.y * (v.y - mp)) + (d.z * (v.z - mp) + d.w * (v.w - mp));
                    } else {
                        a += gp[cv];
                        c2 += gp[cv] * (xp[cv] - mp);
                    }
                }
            }
        }
        if (MODE != 5) a = group_sum(a, lpp);
        if (MODE == 0 || MODE == 1 || MODE == 4) c2 = group_sum(c2, lpp);
        if (gl == 0) {
            if (MODE == 0) {
                m1[hp] = a;
                m2[hp] = c2;
            } else if (MODE == 1) {
                // backward: fold this pixel's own normaliser and statistics into the two maps the
                // transposed window sums need
                float p1 = 0.f, p2 = 0.f;
                if (in) {
                    const float z = norm_at(row, col);
                    const float bc = rsp * rsp * rsp * c2;
                    p1 = (bc * mp - rsp * a) / z;
                    p2 = bc / z;
                }
                m1[hp] = p1;
                m2[hp] = p2;
            } else if (MODE == 4) {
                // gradient of this pixel's variance, divided by its normaliser
                m1[hp] = in ? -0.5f * rsp * rsp * rsp * c2 / norm_at(row, col) : 0.f;
            } else {
                m1[hp] = a;
            }
        }
    }
    __syncthreads();

    // phase 2: window sums, one thread per output pixel
    {
        const int oi = tid / kLcnTile, oj = tid % kLcnTile;
        const int row = ti + oi, col = tj + oj;
        if (row < H && col < W) {
            float s1 = 0.f, s2 = 0.f;
            for (int p = 0; p < ks; ++p)
                for (int q = 0; q < ks; ++q) {
                    const float wt = taps.g[p] * taps.g[q];
                    const int hp = (oi + p) * halo + oj + q;
                    s1 += wt * m1[hp];   // out-of-image halo entries are zero
                    if (kTwoMaps) s2 += wt * m2[hp];
                }
            const size_t pix = img + (size_t)row * W + col;
            if (MODE == 0) {
                const float z = norm_at(row, col);
                const float m = s1 / z, q2 = s2 / z;
                const float var = fmaxf(q2 - m * m, 0.f);
                const float rs = 1.0f / sqrtf(var + eps);
                mu[pix] = m;
                rstd[pix] = rs;
                t1[tid] = m;
                t2[tid] = rs;
            } else if (MODE == 2) {
                mu[pix] = s1 / norm_at(row, col);
            } else if (MODE == 3) {
                const float rs = 1.0f / sqrtf(s1 / norm_at(row, col) + eps);
                rstd[pix] = rs;
                t1[tid] = mu[pix];
                t2[tid] = rs;
            } else {
                t1[tid] = s1;
                t2[tid] = s2;
            }
        }
    }
    if (MODE == 2) return;
    __syncthreads();

    if (MODE == 4) {
        // phase 3 of the two-stage gradient: a pixel's lanes write dv and reduce it over the channels
        for (int op = grp; op < kLcnTile * kLcnTile; op += ngrp) {
            const int oi = op / kLcnTile, oj = op % kLcnTile;
            const int row = ti + oi, col = tj + oj;
            if (row >= H || col >= W) continue;   // uniform over the group
            const size_t pix = img + (size_t)row * W + col;
            const float rs = rstd[pix], m = mu[pix], gs = 2.f * t1[op];
            float acc = 0.f;
            for (int cv = gl; cv < CV; cv += lpp) {
                const size_t o = pix * C + cv * VEC;
                if (VEC == 4) {
                    const float4 xv = *(const float4 *)(x + o), d = *(const float4 *)(dy + o);
                    const float4 g = make_float4(d.x * rs + (xv.x - m) * gs, d.y * rs + (xv.y - m) * gs,
                                                 d.z * rs + (xv.z - m) * gs, d.w * rs + (xv.w - m) * gs);
                    *(float4 *)(out + o) = g;
                    acc += (g.x + g.y) + (g.z + g.w);
                } else {
                    const float g = dy[o] * rs + (x[o] - m) * gs;
                    out[o] = g;
                    acc += g;
                }
            }
            acc = group_sum(acc, lpp);
            if (gl == 0) field[pix] = acc / norm_at(row, col);
        }
        return;
    }

    // phase 3: elementwise pass over the tile
    for (int e = tid; e < kLcnTile * kLcnTile * CV; e += 256) {
        const int cv = e % CV, op = e / CV;
        const int oi = op / kLcnTile, oj = op % kLcnTile;
        const int row = ti + oi, col = tj + oj;
        if (row >= H || col >= W) continue;
        const size_t pix = img + (size_t)row * W + col;
        const size_t o = pix * C + cv * VEC;
        const float u = t1[op], v = t2[op];
        if (MODE == 0 || MODE == 3) {
            if (VEC == 4) {
                const float4 xv = *(const float4 *)(x + o);
                *(float4 *)(out + o) = make_float4((xv.x - u) * v, (xv.y - u) * v, (xv.z - u) * v, (xv.w - u) * v);
            } else {
                out[o] = (x[o] - u) * v;
            }
        } else if (MODE == 1) {
            const float rs = rstd[pix];
            if (VEC == 4) {
                const float4 xv = *(const float4 *)(x + o), d = *(const float4 *)(dy + o);
                *(float4 *)(out + o) = make_float4(d.x * rs + u - xv.x * v, d.y * rs + u - xv.y * v,
                                                   d.z * rs + u - xv.z * v, d.w * rs + u - xv.w * v);
            } else {
                out[o] = dy[o] * rs + u - x[o] * v;
            }
        } else {   // MODE 5
            if (VEC == 4) {
                const float4 d = *(const float4 *)(out + o);
                *(float4 *)(out + o) = make_float4(d.x - u, d.y - u, d.z - u, d.w - u);
            } else {
                out[o] -= u;
            }
        }
    }
}

// Forward pass for C = 4*LPP channels with LPP in {2, 4, 8}: a pixel is exactly one float4 per lane of its group,
// so the tile's own pixels are loaded once, in phase 1, and stay in registers for phase 3; only the halo ring is
// read a second time by the neighbouring tiles.  (The backward pass would keep twice the registers and measured
// slower this way than re-reading the tile.)
template <int LPP>
__global__ __launch_bounds__(256) void lcn_fwd_cached_kernel(const float *__restrict__ x, float *__restrict__ out,
                                                             float *__restrict__ mu, float *__restrict__ rstd, int H,
                                                             int W, int ks, float eps, GaussTaps taps, int tiles_w,
                                                             int tiles_per_img, int zpad) {
    constexpr int C = 4 * LPP, NG = 256 / LPP, NI = LPP;   // NG pixel groups; NI passes cover the 256 tile pixels
    __shared__ float m1[kLcnHalo * kLcnHalo], m2[kLcnHalo * kLcnHalo];
    __shared__ float t1[kLcnTile * kLcnTile], t2[kLcnTile * kLcnTile];
    const int r = (ks - 1) / 2, halo = kLcnTile + 2 * r;
    const int tid = threadIdx.x, grp = tid / LPP, gl = tid % LPP;
    // each XCD walks a contiguous range of tiles: the tiles of one image, whose halos overlap, share an L2
    const int blk = remap_xcd(blockIdx.x, gridDim.x);
    const int b = blk / tiles_per_img, tile = blk - b * tiles_per_img;
    const int ti = (tile / tiles_w) * kLcnTile, tj = (tile % tiles_w) * kLcnTile;
    const size_t img = (size_t)b * H * W;
    // window normalisers of the tile's rows and columns (read after phase 1's barrier)
    __shared__ float zr[kLcnTile], zc[kLcnTile];
    if (tid < kLcnTile) zr[tid] = zpad ? 1.f : tap_norm(taps, ti + tid, H, r);
    else if (tid >= 64 && tid < 64 + kLcnTile) zc[tid - 64] = zpad ? 1.f : tap_norm(taps, tj + tid - 64, W, r);

    // one halo pixel's channel sums -> the two maps of phase 2 (lane 0 of the group writes)
    auto put = [&](int hp, const float4 &v) {
        const float a = group_sum((v.x + v.y) + (v.z + v.w), LPP);
        const float c2 = group_sum((v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w), LPP);
        if (gl == 0) {
            m1[hp] = a;
            m2[hp] = c2;
        }
    };

    // phase 1a: the tile's own pixels, kept in registers (zeros outside the image)
    float4 xv[NI];
    bool inv[NI];
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        const int op = grp + it * NG, oi = op / kLcnTile, oj = op % kLcnTile;
        const int row = ti + oi, col = tj + oj;
        inv[it] = row < H && col < W;
        xv[it] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (inv[it]) xv[it] = *(const float4 *)(x + (img + (size_t)row * W + col) * C + gl * 4);
    }
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        const int op = grp + it * NG, oi = op / kLcnTile, oj = op % kLcnTile;
        put((oi + r) * halo + oj + r, xv[it]);
    }
    // phase 1b: the halo ring around the tile
    for (int hp = grp; hp < halo * halo; hp += NG) {
        const int hi = hp / halo, hj = hp - hi * halo;
        if (hi >= r && hi < r + kLcnTile && hj >= r && hj < r + kLcnTile) continue;   // uniform over the group
        const int row = ti - r + hi, col = tj - r + hj;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row >= 0 && row < H && col >= 0 && col < W) v = *(const float4 *)(x + (img + (size_t)row * W + col) * C + gl * 4);
        put(hp, v);
    }
    __syncthreads();

    // phase 2: window sums and statistics, one thread per output pixel
    {
        const int oi = tid / kLcnTile, oj = tid % kLcnTile;
        const int row = ti + oi, col = tj + oj;
        if (row < H && col < W) {
            float s1 = 0.f, s2 = 0.f;
            for (int p = 0; p < ks; ++p)
                for (int q = 0; q < ks; ++q) {
                    const float wt = taps.g[p] * taps.g[q];
                    const int hp = (oi + p) * halo + oj + q;
                    s1 += wt * m1[hp];   // out-of-image halo entries are zero
                    s2 += wt * m2[hp];
                }
            const float z = zr[oi] * zc[oj] * (float)C;
            const float m = s1 / z, q2 = s2 / z;
            const float var = fmaxf(q2 - m * m, 0.f);
            const float rs = 1.0f / sqrtf(var + eps);
            const size_t pix = img + (size_t)row * W + col;
            mu[pix] = m;
            rstd[pix] = rs;
            t1[tid] = m;
            t2[tid] = rs;
        }
    }
    __syncthreads();

    // phase 3: normalise the registers of phase 1a
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        if (!inv[it]) continue;
        const int op = grp + it * NG, oi = op / kLcnTile, oj = op % kLcnTile;
        const size_t pix = img + (size_t)(ti + oi) * W + tj + oj;
        const float u = t1[op], v = t2[op];
        const float4 xq = xv[it];
        *(float4 *)(out + pix * C + gl * 4) = make_float4((xq.x - u) * v, (xq.y - u) * v, (xq.z - u) * v, (xq.w - u) * v);
    }
}

// Band kernels for the one-stage pooled form, C = 4*LPP channels (LPP a power of two up to 16): a workgroup owns
// RB whole rows of one image.  Its own pixels are loaded once and stay in registers (NV float4 per thread, of x and,
// backward, of dy); only the (ks-1)/2 rows above and below the band are read a second time by the neighbouring
// bands, so a 5x5 window over a band of 22 rows re-reads 18 % of the input where a 16x16 tile re-reads 56 %.
// The maps of per-pixel channel sums carry a margin of (ks-1)/2 zero columns on both sides: phase 2 has no bounds
// checks.  MODE 0: forward (x -> y, mu, rstd).  MODE 1: backward (x, mu, rstd, dy -> dx).
template <int LPP, int MODE, int NTHR, int NV>
__global__ __launch_bounds__(NTHR) void lcn_band_kernel(const float *__restrict__ x, const float *__restrict__ dy,
                                                        float *__restrict__ out, float *__restrict__ mu,
                                                        float *__restrict__ rstd, int H, int W, int ks, float eps,
                                                        GaussTaps taps, int RB, int bands, int zpad, int divx) {
    constexpr int C = 4 * LPP, NH = 2;
    extern __shared__ __attribute__((aligned(16))) float band_lds[];
    const int r = (ks - 1) / 2, MW = W + 2 * r, MH = RB + 2 * r;
    float *m1 = band_lds, *m2 = m1 + MH * MW, *t1 = m2 + MH * MW, *t2 = t1 + RB * W;
    float *zr = t2 + RB * W, *zc = zr + MH;                       // window normalisers of the staged rows, of all columns
    const int tid = threadIdx.x, gl = tid % LPP;
    const int blk = remap_xcd(blockIdx.x, gridDim.x);             // the bands of one image stay in one XCD
    const int b = blk / bands, r0 = (blk - b * bands) * RB;
    const size_t img = (size_t)b * H * W;
    const int npix = RB * W;

    for (int i = tid; i < MH + W; i += NTHR) {
        if (i < MH) zr[i] = zpad ? 1.f : tap_norm(taps, r0 - r + i, H, r);
        else zc[i - MH] = zpad ? 1.f : tap_norm(taps, i - MH, W, r);
    }
    // map cells outside the image are zero; every other cell is written exactly once below
    for (int cell = tid; cell < MH * MW; cell += NTHR) {
        const int hi = cell / MW, hj = cell - hi * MW;
        const int row = r0 - r + hi, col = hj - r;
        if (row < 0 || row >= H || col < 0 || col >= W) m1[cell] = m2[cell] = 0.f;
    }
    if (MODE == 1) __syncthreads();                               // the backward maps use zr and zc

    // channel sums of one pixel (all LPP lanes of its group call this) -> the two maps of phase 2
    auto put = [&](int row, int col, bool in, const float4 &v, const float4 &d) {
        float a, c2;
        float mp = 0.f, rsp = 0.f;
        if (MODE == 0) {
            a = (v.x + v.y) + (v.z + v.w);
            c2 = (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
        } else {
            if (in) { mp = mu[img + (size_t)row * W + col]; rsp = rstd[img + (size_t)row * W + col]; }
            a = (d.x + d.y) + (d.z + d.w);
            c2 = (d.x * (v.x - mp) + d.y * (v.y - mp)) + (d.z * (v.z - mp) + d.w * (v.w - mp));
        }
        a = group_sum(a, LPP);
        c2 = group_sum(c2, LPP);
        if (gl == 0 && in) {
            const int cell = (row - r0 + r) * MW + col + r;
            if (MODE == 0) {
                m1[cell] = a;
                m2[cell] = c2;
            } else {
                // this pixel's own normaliser and statistics folded into what the transposed window sums need
                const float z = zr[row - r0 + r] * zc[col] * (float)C;
                const float bc = rsp * rsp * rsp * c2;
                m1[cell] = (bc * mp - rsp * a) / z;
                m2[cell] = bc / z;
            }
        }
    };

    // phase 1: every load of the workgroup is issued before the first reduction: the band's own pixels, kept in
    // registers, and NH rounds of the rows above and below the band (further rounds, if any, follow)
    float4 xv[NV], dv[MODE == 1 ? NV : 1], hx[NH], hd[MODE == 1 ? NH : 1];
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    const int nhalo = 2 * r * W * LPP;
    auto halo_row = [&](int e) { const int hr = e / (W * LPP); return hr < r ? r0 - r + hr : r0 + RB + hr - r; };
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        const int pp = (q * NTHR + tid) / LPP;
        const int row = r0 + pp / W, col = pp % W;
        xv[q] = zero4;
        if (MODE == 1) dv[q] = zero4;
        if (pp < npix && row < H) {
            const size_t o = (img + (size_t)row * W + col) * C + gl * 4;
            xv[q] = *(const float4 *)(x + o);
            if (MODE == 1) dv[q] = *(const float4 *)(dy + o);
        }
    }
#pragma unroll
    for (int q = 0; q < NH; ++q) {
        const int e = q * NTHR + tid, row = halo_row(e), col = (e / LPP) % W;
        hx[q] = zero4;
        if (MODE == 1) hd[q] = zero4;
        if (e < nhalo && row >= 0 && row < H) {
            const size_t o = (img + (size_t)row * W + col) * C + gl * 4;
            hx[q] = *(const float4 *)(x + o);
            if (MODE == 1) hd[q] = *(const float4 *)(dy + o);
        }
    }
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        const int pp = (q * NTHR + tid) / LPP;
        const int row = r0 + pp / W, col = pp % W;
        put(row, col, pp < npix && row < H, xv[q], MODE == 1 ? dv[q] : zero4);
    }
#pragma unroll
    for (int q = 0; q < NH; ++q) {
        const int e = q * NTHR + tid, row = halo_row(e), col = (e / LPP) % W;
        put(row, col, e < nhalo && row >= 0 && row < H, hx[q], MODE == 1 ? hd[q] : zero4);
    }
    for (int e = NH * NTHR + tid; e < nhalo; e += NTHR) {
        const int row = halo_row(e), col = (e / LPP) % W;
        const bool in = row >= 0 && row < H;
        float4 v = zero4, d = zero4;
        if (in) {
            const size_t o = (img + (size_t)row * W + col) * C + gl * 4;
            v = *(const float4 *)(x + o);
            if (MODE == 1) d = *(const float4 *)(dy + o);
        }
        put(row, col, in, v, d);
    }
    __syncthreads();

    // phase 2: window sums, one thread per pixel of the band
    for (int pp = tid; pp < npix; pp += NTHR) {
        const int oi = pp / W, oj = pp - oi * W, row = r0 + oi;
        if (row >= H) break;
        float s1 = 0.f, s2 = 0.f;
        for (int p = 0; p < ks; ++p) {
            const float *a1 = m1 + (oi + p) * MW + oj, *a2 = m2 + (oi + p) * MW + oj;
            float u1 = 0.f, u2 = 0.f;
            for (int q = 0; q < ks; ++q) {
                u1 += taps.g[q] * a1[q];
                u2 += taps.g[q] * a2[q];
            }
            s1 += taps.g[p] * u1;
            s2 += taps.g[p] * u2;
        }
        if (MODE == 0) {
            const float z = zr[oi + r] * zc[oj] * (float)C;
            const float m = s1 / z, q2 = s2 / z;
            const float rs = 1.0f / sqrtf(fmaxf(q2 - m * m, 0.f) + eps);
            mu[img + (size_t)row * W + oj] = m;
            rstd[img + (size_t)row * W + oj] = rs;
            t1[pp] = m;
            t2[pp] = rs;
        } else {
            t1[pp] = s1;
            t2[pp] = s2;
        }
    }
    __syncthreads();

    // phase 3: elementwise pass over the registers of phase 1a
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        const int pp = (q * NTHR + tid) / LPP;
        const int row = r0 + pp / W, col = pp % W;
        if (pp >= npix || row >= H) continue;
        const size_t pix = img + (size_t)row * W + col;
        const float u = t1[pp], v = t2[pp];
        const float4 xq = xv[q];
        if (MODE == 0) {
            *(float4 *)(out + pix * C + gl * 4) =
                make_float4((xq.x - u) * v, (xq.y - u) * v, (xq.z - u) * v, (xq.w - u) * v);
        } else {
            const float rs = rstd[pix];
            const float4 d = dv[q];
            float4 o = make_float4(d.x * rs + u - xq.x * v, d.y * rs + u - xq.y * v, d.z * rs + u - xq.z * v,
                                   d.w * rs + u - xq.w * v);
            // divx: the gradient divided by x itself, which is what the backward pass of a pooling layer in front
            // of this one sums up (x is that layer's output, positive)
            if (divx) o = make_float4(o.x / xq.x, o.y / xq.y, o.z / xq.z, o.w / xq.w);
            *(float4 *)(out + pix * C + gl * 4) = o;
        }
    }
}

// Fused forward pass: 3x3 stride-1 L2 pooling, then the one-stage pooled LCN of the pooled map, which is written out
// as well (the backward passes need it).  x [B,H,W,C] -> p [B,H-2,W-2,C] -> y, mu, rstd; C = 4*LPP.
// A workgroup owns PB whole rows of p of one image (plus the (ks-1)/2 rows above and below them, which the
// neighbouring bands compute a second time).  Pooling: a wave covers 64/LPP consecutive columns of x and walks down
// rpt + 2 rows; a lane squares its own pixels (every x value the workgroup needs is loaded exactly once, all loads in
// flight together), adds three rows at a time in registers and takes the two columns to its right from the lanes
// LPP and 2 LPP further on, so a wave produces 64/LPP - 2 columns of p.  WPS such waves cover a row; the 16 waves
// are 16/WPS segments of rpt rows each.  The pooled values stay in registers (at most RPT float4 per lane); their
// channel sums go into the LDS maps, and the rest is the band kernel's phases 2 and 3.
template <int LPP, int RPT>
__global__ __launch_bounds__(kBandThreads) void pool_lcn_band_kernel(const float *__restrict__ x, float *__restrict__ p,
                                                                     float *__restrict__ out, float *__restrict__ mu,
                                                                     float *__restrict__ rstd, int H, int W, int ks,
                                                                     float peps, float eps, GaussTaps taps, int PB,
                                                                     int bands, int WPS, int rpt) {
    constexpr int C = 4 * LPP, CPW = 64 / LPP, OPW = CPW - 2, NTHR = kBandThreads;
    extern __shared__ __attribute__((aligned(16))) float band_lds[];
    const int Hp = H - 2, Wp = W - 2;
    const int r = (ks - 1) / 2, MW = Wp + 2 * r, MH = PB + 2 * r;
    float *m1 = band_lds, *m2 = m1 + MH * MW, *t1 = m2 + MH * MW, *t2 = t1 + PB * Wp;
    float *zr = t2 + PB * Wp, *zc = zr + MH, *tg = zc + Wp;     // tg: the taps (indexed by loop counters below)
    // the wave index as a scalar: every row index below is then scalar too, and a row's address is a scalar base
    // plus one lane offset that all rows share
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int gl = lane % LPP, cw = lane / LPP;
    const int seg = wave / WPS, ws = wave - seg * WPS;
    const int blk = remap_xcd(blockIdx.x, gridDim.x);
    const int b = blk / bands, r0 = (blk - b * bands) * PB;
    const size_t ximg = (size_t)b * H * W, pimg = (size_t)b * Hp * Wp;

    for (int i = tid; i < MH + Wp; i += NTHR) {
        if (i < MH) zr[i] = tap_norm(taps, r0 - r + i, Hp, r);
        else zc[i - MH] = tap_norm(taps, i - MH, Wp, r);
    }
    if (tid < kLcnMaxK) tg[tid] = taps.g[tid];
    // map cells outside the pooled image are zero; every other cell is written exactly once below
    for (int cell = tid; cell < MH * MW; cell += NTHR) {
        const int hi = cell / MW, hj = cell - hi * MW;
        const int row = r0 - r + hi, col = hj - r;
        if (row < 0 || row >= Hp || col < 0 || col >= Wp) m1[cell] = m2[cell] = 0.f;
    }

    // pooling: staged row hrow of the band is row r0 - r + hrow of p and needs rows r0 - r + hrow .. + 2 of x
    const int col = ws * OPW + cw;          // column of x this lane loads = column of p it produces
    const int hrow0 = seg * rpt;
    const int xoff = min(col, W - 1) * C + gl * 4, poff = min(col, Wp - 1) * C + gl * 4;
    f32x4 q[RPT + 2];
#pragma unroll
    for (int t = 0; t < RPT + 2; ++t) {
        // every lane loads, from an address clamped into the image; what lies outside counts as zero
        const int xrow = r0 - r + hrow0 + t;
        const bool in = t < rpt + 2 && hrow0 < MH && xrow >= 0 && xrow < H && col < W;
        const float *rowp = x + (ximg + (size_t)min(max(xrow, 0), H - 1) * W) * C;
        const f32x4 v = *(const f32x4 *)(rowp + xoff);
        q[t] = in ? v : (f32x4){0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int t = 0; t < RPT + 2; ++t) q[t] *= q[t];
#pragma unroll
    for (int t = 0; t < RPT; ++t) {
        const f32x4 v = (q[t] + q[t + 1]) + q[t + 2];
        f32x4 o;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            o[c] = __builtin_amdgcn_sqrtf(peps + ((v[c] + __shfl_down(v[c], LPP, 64)) + __shfl_down(v[c], 2 * LPP, 64)));
        q[t] = o;                            // p[hrow0 + t][col], valid for cw < OPW
        // one row's cross-lane reads at a time (the next row's input is tied to this row's result): with all of
        // them in flight the results alone fill the registers
        asm volatile("" : "+v"(q[t + 1][0]), "+v"(q[t + 1][1]), "+v"(q[t + 1][2]), "+v"(q[t + 1][3]) : "v"(o[0]), "v"(o[1]), "v"(o[2]), "v"(o[3]));
    }
    // channel sums of the pooled pixels -> the two maps of phase 2 (all lanes take part in the reductions)
#pragma unroll
    for (int t = 0; t < RPT; ++t) {
        const int hrow = hrow0 + t, prow = r0 - r + hrow;
        const f32x4 v = q[t];
        float a = (v[0] + v[1]) + (v[2] + v[3]);
        float c2 = (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
        a = group_sum(a, LPP);
        c2 = group_sum(c2, LPP);
        if (gl == 0 && t < rpt && hrow < MH && prow >= 0 && prow < Hp && cw < OPW && col < Wp) {
            const int cell = hrow * MW + col + r;
            m1[cell] = a;
            m2[cell] = c2;
        }
    }
    __syncthreads();

    // phase 2: window sums, one thread per pixel of the band
    for (int pp = tid; pp < PB * Wp; pp += NTHR) {
        const int oi = pp / Wp, oj = pp - oi * Wp, row = r0 + oi;
        if (row >= Hp) break;
        float s1 = 0.f, s2 = 0.f;
        for (int a = 0; a < ks; ++a) {
            const float *a1 = m1 + (oi + a) * MW + oj, *a2 = m2 + (oi + a) * MW + oj;
            float u1 = 0.f, u2 = 0.f;
            for (int c = 0; c < ks; ++c) {
                u1 += tg[c] * a1[c];
                u2 += tg[c] * a2[c];
            }
            s1 += tg[a] * u1;
            s2 += tg[a] * u2;
        }
        const float z = zr[oi + r] * zc[oj] * (float)C;
        const float m = s1 / z, q2 = s2 / z;
        const float rs = 1.0f / sqrtf(fmaxf(q2 - m * m, 0.f) + eps);
        mu[pimg + (size_t)row * Wp + oj] = m;
        rstd[pimg + (size_t)row * Wp + oj] = rs;
        t1[pp] = m;
        t2[pp] = rs;
    }
    __syncthreads();

    // phase 3: the band's own rows: p and the normalised values
#pragma unroll
    for (int t = 0; t < RPT; ++t) {
        const int prow = r0 - r + hrow0 + t;
        if (t >= rpt || prow < r0 || prow >= r0 + PB || prow >= Hp || cw >= OPW || col >= Wp) continue;
        const int pp = (prow - r0) * Wp + col;
        const float u = t1[pp], v = t2[pp];
        const size_t o = (pimg + (size_t)prow * Wp) * C;
        *(f32x4 *)(p + o + poff) = q[t];
        *(f32x4 *)(out + o + poff) = (f32x4){(q[t][0] - u) * v, (q[t][1] - u) * v, (q[t][2] - u) * v, (q[t][3] - u) * v};
    }
}

namespace {

int grid_for(long long total) {
    long long blocks = (total + 255) / 256;
    const long long cap = 256LL * 32;  // 32 workgroups per compute unit, grid-stride beyond that
    return (int)(blocks < cap ? (blocks > 0 ? blocks : 1) : cap);
}

bool make_taps(int ks, float sigma, GaussTaps *t) {
    if (ks < 1 || ks > kLcnMaxK || (ks & 1) == 0 || !(sigma > 0.f)) return false;
    const int r = (ks - 1) / 2;
    double s = 0.0, g[kLcnMaxK];
    for (int p = -r; p <= r; ++p) {
        g[p + r] = exp(-(double)(p * p) / (2.0 * (double)sigma * (double)sigma));
        s += g[p + r];
    }
    for (int p = 0; p < kLcnMaxK; ++p) t->g[p] = p < ks ? (float)(g[p] / s) : 0.f;
    return true;
}

int lanes_per_pixel(int cv) {
    int l = 1;
    while (l < cv && l < 64) l <<= 1;
    return l;
}

}  // namespace

int launch_l2pool_fwd(const float *x, float *y, int B, int H, int W, int C, int ks, int st, float eps,
                      hipStream_t s) {
    const int Ho = (H - ks) / st + 1, Wo = (W - ks) / st + 1;
    const size_t patch_bytes = (size_t)(kPoolTH + ks - 1) * (kPoolTW + ks - 1) * C * sizeof(float);
    if (C % 4 == 0 && st == 1 && ks == 3 && Ho > 0 && Wo > 0 && B > 0) {
        // segments of RS rows, a multiple of the four rows a thread has in flight: enough segments for about
        // sixteen waves per compute unit (48 x 48 x 32 maps, batch 128: 8 rows 11.7 us, 4 rows 12.1 us, 16 rows 13.5 us)
        const int CV = C / 4;
        const long long cols = (long long)B * Wo * CV;
        const long long want = std::max<long long>((256LL * 16 * 64 + cols - 1) / cols, 1);
        const int RS = (int)std::max<long long>(((Ho + want - 1) / want + 3) / 4 * 4, 4);
        const int nseg = (Ho + RS - 1) / RS;
        const long long total = cols * nseg, nblk = (total + 255) / 256;
        if (nblk > 0x7fffffffLL) return LC_EUNSUPPORTED;
        hipLaunchKernelGGL((l2pool_fwd_stream_kernel<3, 4>), dim3((unsigned)nblk), dim3(256), 0, s, x, y, H, W, CV, Ho,
                           Wo, RS, nseg, eps, total);
    } else if (C % 4 == 0 && st == 1 && ks <= kPoolMaxK && patch_bytes <= 64 * 1024) {
        const int th = (Ho + kPoolTH - 1) / kPoolTH, tw = (Wo + kPoolTW - 1) / kPoolTW;
        const long long nblk = (long long)B * th * tw;
        if (nblk > 0x7fffffffLL) return LC_EUNSUPPORTED;
        auto kern = l2pool_tile_kernel<0>;
        if (int rc_lds = allow_dynamic_lds((const void *)kern, patch_bytes, "l2pool_fwd: hipFuncSetAttribute")) return rc_lds;
        hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(256), patch_bytes, s, x, (const float *)nullptr,
                           (const float *)nullptr, y, H, W, C, Ho, Wo, ks, eps, tw, th * tw);
    } else if (C % 4 == 0 && st == 1 && ks <= kPoolMaxK && B <= 65535 && (long long)H * W * C < (1LL << 30)) {
        const int groups = (Wo + kPoolOW - 1) / kPoolOW;
        hipLaunchKernelGGL(l2pool_fwd_rows_kernel, dim3((Ho * groups * (C / 4) + 255) / 256, B), dim3(256), 0, s, x, y, H,
                           W, C, Ho, Wo, ks, eps, groups);
    } else if (C % 4 == 0) {
        const long long total = (long long)B * Ho * Wo * (C / 4);
        hipLaunchKernelGGL(l2pool_fwd_kernel<4>, dim3(grid_for(total)), dim3(256), 0, s, x, y, B, H, W, C, Ho, Wo, ks,
                           st, eps, total);
    } else {
        const long long total = (long long)B * Ho * Wo * C;
        hipLaunchKernelGGL(l2pool_fwd_kernel<1>, dim3(grid_for(total)), dim3(256), 0, s, x, y, B, H, W, C, Ho, Wo, ks,
                           st, eps, total);
    }
    LC_HIP_LAUNCH_CHECK("l2pool_fwd launch");
    return LC_OK;
}

int launch_l2pool_bwd(const float *x, const float *y, const float *dy, float *dx, int B, int H, int W, int C, int ks,
                      int st, hipStream_t s) {
    const int Ho = (H - ks) / st + 1, Wo = (W - ks) / st + 1;
    const size_t patch_bytes = (size_t)(kPoolTH + ks - 1) * (kPoolTW + ks - 1) * C * sizeof(float);
    if (C % 4 == 0 && st == 1 && ks <= kPoolMaxK && patch_bytes <= 64 * 1024) {
        const int th = (H + kPoolTH - 1) / kPoolTH, tw = (W + kPoolTW - 1) / kPoolTW;
        const long long nblk = (long long)B * th * tw;
        if (nblk > 0x7fffffffLL) return LC_EUNSUPPORTED;
        auto kern = l2pool_tile_kernel<1>;
        if (int rc_lds = allow_dynamic_lds((const void *)kern, patch_bytes, "l2pool_bwd: hipFuncSetAttribute")) return rc_lds;
        hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(256), patch_bytes, s, x, y, dy, dx, H, W, C, Ho, Wo, ks,
                           0.f, tw, th * tw);
    } else if (C % 4 == 0 && st == 1 && ks <= kPoolMaxK && B <= 65535 && (long long)H * W * C < (1LL << 30)) {
        const int groups = (W + kPoolOW - 1) / kPoolOW;
        hipLaunchKernelGGL(l2pool_bwd_rows_kernel, dim3((H * groups * (C / 4) + 255) / 256, B), dim3(256), 0, s, x, y, dy,
                           dx, H, W, C, Ho, Wo, ks, groups);
    } else if (C % 4 == 0) {
        const long long total = (long long)B * H * W * (C / 4);
        hipLaunchKernelGGL(l2pool_bwd_kernel<4>, dim3(grid_for(total)), dim3(256), 0, s, x, y, dy, dx, B, H, W, C, Ho,
                           Wo, ks, st, total);
    } else {
        const long long total = (long long)B * H * W * C;
        hipLaunchKernelGGL(l2pool_bwd_kernel<1>, dim3(grid_for(total)), dim3(256), 0, s, x, y, dy, dx, B, H, W, C, Ho,
                           Wo, ks, st, total);
    }
    LC_HIP_LAUNCH_CHECK("l2pool_bwd launch");
    return LC_OK;
}

namespace {

// Rows per band: as many as the registers hold (NV float4 per thread), split evenly over the image.  The band
// kernel pays where a band is at least 8 rows and two window radii high; below that the 16x16 tiles re-read less.
template <int LPP, int MODE>
int launch_lcn_band_lpp(const float *x, const float *dy, float *out, float *mu, float *rstd, int B, int H, int W,
                        int ks, float eps, const GaussTaps &taps, hipStream_t s, int zero_pad, bool *done, int divx) {
    constexpr int NTHR = kBandThreads, NV = 8;
    const int r = (ks - 1) / 2;
    const int rb_max = (NTHR * NV) / (W * LPP);
    if (rb_max < 8 || rb_max < 2 * r) return LC_OK;
    const int bands = (H + rb_max - 1) / rb_max, RB = (H + bands - 1) / bands;
    const size_t lds = ((size_t)2 * (RB + 2 * r) * (W + 2 * r) + (size_t)2 * RB * W + (RB + 2 * r) + W) * sizeof(float);
    const long long nblk = (long long)B * bands;
    if (lds > 64 * 1024 || nblk > 0x7fffffffLL) return LC_OK;
    auto kern = lcn_band_kernel<LPP, MODE, NTHR, NV>;
    if (int rc_lds = allow_dynamic_lds((const void *)kern, lds, "lcn: hipFuncSetAttribute")) return rc_lds;
    *done = true;
    hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(NTHR), lds, s, x, dy, out, mu, rstd, H, W, ks, eps, taps, RB,
                       bands, zero_pad, divx);
    LC_HIP_LAUNCH_CHECK("lcn launch");
    return LC_OK;
}

int launch_lcn_band(int mode, const float *x, const float *dy, float *out, float *mu, float *rstd, int B, int H, int W,
                    int C, int ks, float eps, const GaussTaps &taps, hipStream_t s, int zero_pad, bool *done,
                    int divx = 0) {
#define LC_BAND(LPP_)                                                                                                  \
    return mode == 0 ? launch_lcn_band_lpp<LPP_, 0>(x, dy, out, mu, rstd, B, H, W, ks, eps, taps, s, zero_pad, done, 0) \
                     : launch_lcn_band_lpp<LPP_, 1>(x, dy, out, mu, rstd, B, H, W, ks, eps, taps, s, zero_pad, done, divx)
    switch (C) {
        case 4: LC_BAND(1);
        case 8: LC_BAND(2);
        case 16: LC_BAND(4);
        case 32: LC_BAND(8);
        case 64: LC_BAND(16);
        default: return LC_OK;
    }
#undef LC_BAND
}

}  // namespace

namespace {

template <int LPP, int RPT>
int launch_pool_lcn_band(const LaunchPlan &plan, const float *x, float *p, float *out, float *mu, float *rstd, int H,
                         int W, int ks, float peps, float eps, const GaussTaps &taps, int PB, int bands, int WPS,
                         int rpt, hipStream_t s) {
    auto kern = pool_lcn_band_kernel<LPP, RPT>;
    LC_LAUNCH(plan, "l2pool_lcn_fwd launch", kern, s, x, p, out, mu, rstd, H, W, ks, peps, eps, taps, PB, bands, WPS,
              rpt);
    return LC_OK;
}

}  // namespace

// Gradient of l2pool_lcn_fwd with respect to its input: lcn_bwd, then l2pool_bwd, with `scratch` ([B,Ho,Wo,C]) between
// them.  Where the band kernel and the tile kernel apply, the first leaves its gradient already divided by p there,
// so the second reads one array less.
int launch_lcn_pool_bwd(const float *x, const float *p, const float *mu, const float *rstd, const float *dn,
                        float *scratch, float *dx, int B, int H, int W, int C, int pks, int pst, int ks, float sigma,
                        hipStream_t s) {
    const int Ho = (H - pks) / pst + 1, Wo = (W - pks) / pst + 1;
    GaussTaps taps;
    if (!make_taps(ks, sigma, &taps)) return LC_EINVAL;
    const size_t patch_bytes = (size_t)(kPoolTH + pks - 1) * (kPoolTW + pks - 1) * C * sizeof(float);
    const int th = (H + kPoolTH - 1) / kPoolTH, tw = (W + kPoolTW - 1) / kPoolTW;
    const long long nblk = (long long)B * th * tw;
    if (C % 4 == 0 && pst == 1 && pks <= kPoolMaxK && patch_bytes <= 64 * 1024 && nblk <= 0x7fffffffLL) {
        bool done = false;
        if (int rc = launch_lcn_band(1, p, dn, scratch, const_cast<float *>(mu), const_cast<float *>(rstd), B, Ho, Wo, C,
                                     ks, 0.f, taps, s, 0, &done, 1))
            return rc;
        if (done) {
            auto kern = l2pool_tile_kernel<2>;
            if (int rc_lds = allow_dynamic_lds((const void *)kern, patch_bytes, "lcn_l2pool_bwd: hipFuncSetAttribute"))
                return rc_lds;
            hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(256), patch_bytes, s, x, (const float *)nullptr,
                               (const float *)scratch, dx, H, W, C, Ho, Wo, pks, 0.f, tw, th * tw);
            LC_HIP_LAUNCH_CHECK("lcn_l2pool_bwd launch");
            return LC_OK;
        }
    }
    if (int rc = launch_lcn(1, p, dn, scratch, const_cast<float *>(mu), const_cast<float *>(rstd), B, Ho, Wo, C, ks, sigma,
                            0.f, s))
        return rc;
    return launch_l2pool_bwd(x, p, scratch, dx, B, H, W, C, pks, pst, s);
}

// Host check of a pool_lcn_band_kernel launch.  tparam = {LPP, RPT}; arg = {PB, bands, WPS, rpt, H, W, ks, B}.
int check_pool_lcn_band(const LaunchPlan &p) {
    const int LPP = p.tparam[0], RPT = p.tparam[1];
    const int PB = p.arg[0], bands = p.arg[1], WPS = p.arg[2], rpt = p.arg[3], H = p.arg[4], W = p.arg[5], ks = p.arg[6];
    const int B = p.arg[7];
    const int Hp = H - 2, Wp = W - 2, r = (ks - 1) / 2, MH = PB + 2 * r, MW = Wp + 2 * r;
    LC_PLAN_REQUIRE(p, (int)p.block == kBandThreads && (LPP == 2 || LPP == 4 || LPP == 8 || LPP == 16));
    LC_PLAN_REQUIRE(p, Hp >= 1 && Wp >= 1 && PB >= 1 && bands >= 1 && (long long)PB * bands >= Hp);
    // the waves of a segment cover a row of p, the segments cover the band and its halo rows, a lane's rows fit
    const int OPW = 64 / LPP - 2;
    LC_PLAN_REQUIRE(p, WPS >= 1 && WPS <= 16 && WPS * OPW >= Wp);
    LC_PLAN_REQUIRE(p, rpt >= 1 && rpt <= RPT && (16 / WPS) * rpt >= MH);
    LC_PLAN_REQUIRE(p, p.lds_bytes >= ((size_t)2 * MH * MW + (size_t)2 * PB * Wp + MH + Wp + kLcnMaxK) * sizeof(float));
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] == (long long)B * bands && p.grid[1] == 1 && p.grid[2] == 1);
    return LC_OK;
}

// Fused pooling + LCN forward for 3x3 stride-1 pooling and 8, 16, 32 or 64 channels, where a row of the pooled map
// fits the 16 waves of a workgroup; *done tells whether it was launched.
int launch_pool_lcn_fused(const float *x, float *p, float *out, float *mu, float *rstd, int B, int H, int W, int C,
                          float peps, int ks, float sigma, float eps, hipStream_t s, bool *done) {
    *done = false;
    GaussTaps taps;
    if (!make_taps(ks, sigma, &taps)) return LC_EINVAL;
    const int LPP = C / 4, Hp = H - 2, Wp = W - 2, r = (ks - 1) / 2;
    if (C % 4 != 0 || (LPP != 2 && LPP != 4 && LPP != 8 && LPP != 16) || Hp < 1 || Wp < 1) return LC_OK;
    const int OPW = 64 / LPP - 2, WPS = (Wp + OPW - 1) / OPW;
    if (WPS > 16) return LC_OK;
    const int nseg = 16 / WPS;
    // bands per image: enough for one workgroup per compute unit (twice as many measured the same or slower: 25.0
    // against 26.3 us on 128 x 46 x 46 x 32 maps, 13.1 against 10.8 us on 128 x 25 x 25 x 32), and as many more as it
    // takes for a lane's rows to fit its registers and the band's maps 64 KB of LDS
    int bands = std::min(Hp, std::max(1, (256 + B - 1) / B)), PB = 0, rpt = 0;
    size_t lds = 0;
    for (;; ++bands) {
        PB = (Hp + bands - 1) / bands;
        rpt = (PB + 2 * r + nseg - 1) / nseg;
        lds = ((size_t)2 * (PB + 2 * r) * (Wp + 2 * r) + (size_t)2 * PB * Wp + (PB + 2 * r) + Wp + kLcnMaxK) * sizeof(float);
        if ((rpt <= 13 && lds <= 64 * 1024) || bands >= Hp) break;
    }
    if (rpt > 13 || lds > 64 * 1024) return LC_OK;
    bands = (Hp + PB - 1) / PB;
    if ((long long)B * bands > 0x7fffffffLL) return LC_OK;
    const int RPT = rpt <= 4 ? 4 : rpt <= 8 ? 8 : 13;
    const LaunchPlan plan = make_plan("pool_lcn_band", {LPP, RPT}, {PB, bands, WPS, rpt, H, W, ks, B},
                                      dim3((unsigned)(B * bands)), kBandThreads, lds);
    if (int rc = check_pool_lcn_band(plan)) return rc;
    *done = true;
#define LC_PLB(LPP_, RPT_) \
    return launch_pool_lcn_band<LPP_, RPT_>(plan, x, p, out, mu, rstd, H, W, ks, peps, eps, taps, PB, bands, WPS, rpt, s)
#define LC_PLB_R(LPP_) do { if (RPT == 4) LC_PLB(LPP_, 4); if (RPT == 8) LC_PLB(LPP_, 8); LC_PLB(LPP_, 13); } while (0)
    switch (LPP) {
        case 2: LC_PLB_R(2);
        case 4: LC_PLB_R(4);
        case 8: LC_PLB_R(8);
        default: LC_PLB_R(16);
    }
#undef LC_PLB_R
#undef LC_PLB
}

int launch_lcn(int mode, const float *x, const float *dy, float *out, float *mu, float *rstd, int B, int H, int W,
               int C, int ks, float sigma, float eps, hipStream_t s, int zero_pad, float *field) {
    GaussTaps taps;
    if (!make_taps(ks, sigma, &taps)) return LC_EINVAL;
    if (mode < 0 || mode > 5 || ((mode == 4 || mode == 5) && field == nullptr)) return LC_EINVAL;
    const int tiles_h = (H + kLcnTile - 1) / kLcnTile, tiles_w = (W + kLcnTile - 1) / kLcnTile;
    const long long nblk = (long long)B * tiles_h * tiles_w;
    if (nblk > 0x7fffffffLL) return LC_EUNSUPPORTED;
    if (mode == 0 || mode == 1) {
        bool done = false;
        const int rc = launch_lcn_band(mode, x, dy, out, mu, rstd, B, H, W, C, ks, eps, taps, s, zero_pad, &done);
        if (done) return rc;
    }
    const int vec = (C % 4 == 0) ? 4 : 1;
    const int lpp = lanes_per_pixel(C / vec);
    dim3 grid((unsigned)nblk), block(256);
#define LC_LCN(VEC_, MODE_)                                                                                      \
    hipLaunchKernelGGL((lcn_kernel<VEC_, MODE_>), grid, block, 0, s, x, dy, out, mu, rstd, field, H, W, C, ks, eps, \
                       taps, lpp, tiles_w, tiles_h * tiles_w, zero_pad)
#define LC_LCN_MODE(MODE_) do { if (vec == 4) LC_LCN(4, MODE_); else LC_LCN(1, MODE_); } while (0)
#define LC_LCN_CACHED(LPP_)                                                                                    \
    hipLaunchKernelGGL((lcn_fwd_cached_kernel<LPP_>), grid, block, 0, s, x, out, mu, rstd, H, W, ks, eps, taps, \
                       tiles_w, tiles_h * tiles_w, zero_pad)
    if (mode == 0 && C == 32) LC_LCN_CACHED(8);
    else if (mode == 0 && C == 16) LC_LCN_CACHED(4);
    else if (mode == 0 && C == 8) LC_LCN_CACHED(2);
    else if (mode == 0) LC_LCN_MODE(0);
    else if (mode == 1) LC_LCN_MODE(1);
    else if (mode == 2) LC_LCN_MODE(2);
    else if (mode == 3) LC_LCN_MODE(3);
    else if (mode == 4) LC_LCN_MODE(4);
    else LC_LCN_MODE(5);
#undef LC_LCN_CACHED
#undef LC_LCN_MODE
#undef LC_LCN
    LC_HIP_LAUNCH_CHECK("lcn launch");
    return LC_OK;
}

}  // namespace lc
