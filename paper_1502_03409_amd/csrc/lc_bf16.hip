// bf16-operand, fp32-accumulate variants of the three layer contractions (x, w, dy stored as bf16;
// y, dx, dw fp32).  Same mathematics and layouts as the fp32 kernels (Eq. 1 / Sec. 3.1 geometry).
//
// All three use v_mfma_f32_16x16x16_bf16: lane (i, kk) of an operand holds four consecutive
// contraction indices 4kk..4kk+3 of row/column i.  Where the contraction index is contiguous in memory
// (backward data: f) a lane's four values are one 8-byte load.  Where it is the strided index (forward:
// k of w[k][f]; backward weights: the batch) a lane loads four rows of four consecutive free indices
// and transposes the 4x4 block in registers (v_perm_b32): it then owns column i of four different
// tiles, free index 4i+u in tile u, and 16 lanes still cover whole 128-byte lines.
// Waves are independent (no LDS); loads run one or two steps ahead in a register ring.
#include "lc_common.hpp"

namespace lc {

typedef const __attribute__((address_space(1))) u32x2 *g2_ptr;
typedef const __attribute__((address_space(1))) unsigned short *gh_ptr;

// r[t] = four bf16 (e0..e3) of row t.  o[u] = (r[0].e_u, r[1].e_u, r[2].e_u, r[3].e_u).
__device__ __forceinline__ void transpose4x4_bf16(const u32x2 (&r)[4], u32x2 (&o)[4]) {
    constexpr unsigned LO = 0x05040100u, HI = 0x07060302u;   // low / high halves of {src0:src1}
    o[0] = (u32x2){__builtin_amdgcn_perm(r[1][0], r[0][0], LO), __builtin_amdgcn_perm(r[3][0], r[2][0], LO)};
    o[1] = (u32x2){__builtin_amdgcn_perm(r[1][0], r[0][0], HI), __builtin_amdgcn_perm(r[3][0], r[2][0], HI)};
    o[2] = (u32x2){__builtin_amdgcn_perm(r[1][1], r[0][1], LO), __builtin_amdgcn_perm(r[3][1], r[2][1], LO)};
    o[3] = (u32x2){__builtin_amdgcn_perm(r[1][1], r[0][1], HI), __builtin_amdgcn_perm(r[3][1], r[2][1], HI)};
}

// ------------------------------------------------------------------------------------ forward
// wave task = (location, 64 filters, 16*MT images).  Contraction step = 16 patch elements.
template <int MT>
__global__ __launch_bounds__(256) void lc_forward_bf16_kernel(Geom g, const unsigned short *__restrict__ x,
                                                              const unsigned short *__restrict__ w,
                                                              const float *__restrict__ bias, float alpha,
                                                              float *__restrict__ y, int fblocks, int btiles,
                                                              int ntasks) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kk = lane >> 4;
    const int task = remap_xcd(blockIdx.x, gridDim.x) * 4 + wave;
    if (task >= ntasks) return;
    const int per_loc = fblocks * btiles;
    const int loc = task / per_loc, rest = task - loc * per_loc;
    const int f0 = (rest / btiles) * 64, b0 = (rest % btiles) * 16 * MT;
    const int i = loc / g.LW, j = loc - i * g.LW;
    const size_t img = (size_t)g.H * g.W * g.C;

    f32x4 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[mt][u] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // images of this lane (rows of A); rows beyond the batch read image B-1 and are never stored
    gh_ptr xa[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int b = min(b0 + mt * 16 + n, g.B - 1);
        xa[mt] = (gh_ptr)x + (size_t)b * img + ((size_t)(i * g.S) * g.W + j * g.S) * g.C;
    }
    gh_ptr wl = (gh_ptr)w + (size_t)loc * g.K * g.F + f0 + 4 * n;
    const int WC = g.W * g.C;
    for (int kh = 0; kh < g.R; ++kh) {
        for (int q0 = 0; q0 < g.RC; q0 += 16) {          // RC % 16 == 0 on this path
            const int q = q0 + 4 * kk, k = kh * g.RC + q;
            u32x2 r[4], bo[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) r[t] = *(g2_ptr)(wl + (size_t)(k + t) * g.F);
            u32x2 a[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[mt] = *(g2_ptr)(xa[mt] + kh * WC + q);
            transpose4x4_bf16(r, bo);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int u = 0; u < 4; ++u) acc[mt][u] = mfma16_bf16(a[mt], bo[u], acc[mt][u]);
        }
    }
    f32x4 bv = (f32x4){0.f, 0.f, 0.f, 0.f};
    if (bias) bv = *(const f32x4 *)(bias + (size_t)loc * g.F + f0 + 4 * n);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int b = b0 + mt * 16 + 4 * kk + rr;
            if (b >= g.B) continue;
            f32x4 o;
#pragma unroll
            for (int u = 0; u < 4; ++u) o[u] = alpha * acc[mt][u][rr] + bv[u];
            *(f32x4 *)(y + ((size_t)b * g.L + loc) * g.F + f0 + 4 * n) = o;
        }
}

// ------------------------------------------------------------------------------ backward data
// wave task = (cell, 64 cell values, 16*MT images); contraction over (a, a', f), 16 f per step.
template <int MT>
__global__ __launch_bounds__(256) void lc_bwd_data_bf16_kernel(Geom g, const unsigned short *__restrict__ dy,
                                                               const unsigned short *__restrict__ w,
                                                               float *__restrict__ dx, int CW, int nblocks,
                                                               int btiles, int ntasks) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, kk = lane >> 4;
    const int task = remap_xcd(blockIdx.x, gridDim.x) * 4 + wave;
    if (task >= ntasks) return;
    const int per_cell = nblocks * btiles;
    const int cell = task / per_cell, rest = task - cell * per_cell;
    const int n0 = (rest / btiles) * 64, b0 = (rest % btiles) * 16 * MT;
    const int ri = cell / CW, wi = cell - ri * CW;
    const int SC = g.S * g.C, NCV = g.S * SC, AP = g.R / g.S;

    int kn[4];          // offset of this lane's cell value inside a field's K x F matrix, per N-tile
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        const int nn = n0 + nt * 16 + m;
        const int nc = nn < NCV ? nn : 0;
        const int dr = nc / SC;
        kn[nt] = (dr * g.RC + (nc - dr * SC)) * g.F + 4 * kk;
    }
    f32x4 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const size_t dyimg = (size_t)g.L * g.F;
    gh_ptr da[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) da[mt] = (gh_ptr)dy + (size_t)min(b0 + mt * 16 + m, g.B - 1) * dyimg + 4 * kk;

    for (int a = 0; a < AP; ++a) {
        const int i = ri - a;
        if (i < 0 || i >= g.LH) continue;
        for (int ap = 0; ap < AP; ++ap) {
            const int j = wi - ap;
            if (j < 0 || j >= g.LW) continue;
            const size_t loc = (size_t)i * g.LW + j;
            gh_ptr wl = (gh_ptr)w + (loc * g.K + (size_t)g.S * a * g.RC + g.S * ap * g.C) * g.F;
            for (int f = 0; f < g.F; f += 16) {          // F % 16 == 0 on this path
                u32x2 bo[4], av[MT];
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) bo[nt] = *(g2_ptr)(wl + kn[nt] + f);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) av[mt] = *(g2_ptr)(da[mt] + loc * g.F + f);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = mfma16_bf16(av[mt], bo[nt], acc[mt][nt]);
            }
        }
    }
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        const int nn = n0 + nt * 16 + m;
        if (nn >= NCV) continue;
        const int dr = nn / SC, rem = nn - dr * SC;
        const int row = ri * g.S + dr, col = wi * g.S + rem / g.C;
        if (row >= g.H || col >= g.W) continue;
        const size_t pix = ((size_t)row * g.W + wi * g.S) * g.C + rem;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int b = b0 + mt * 16 + 4 * kk + r;
                if (b < g.B) dx[(size_t)b * g.H * g.W * g.C + pix] = acc[mt][nt][r];
            }
    }
}

// --------------------------------------------------------------------------- backward weights
// wave task = (location, 128 patch elements) x 64 filters; contraction over the batch, 16 images per step.
__global__ __launch_bounds__(256) void lc_bwd_weights_bf16_kernel(Geom g, const unsigned short *__restrict__ x,
                                                                  const unsigned short *__restrict__ dy, float beta,
                                                                  float *__restrict__ out, int kblocks, int ntasks) {
    constexpr int G = 2;                      // groups of 4 M-tiles: 128 patch elements per task
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, kk = lane >> 4;
    const int task = remap_xcd(blockIdx.x, gridDim.x) * 4 + wave;
    if (task >= ntasks) return;
    const int loc = task / kblocks, k0 = (task - loc * kblocks) * (G * 64);
    const int i = loc / g.LW, j = loc - i * g.LW;
    const int f0 = blockIdx.y * 64;
    const size_t img = (size_t)g.H * g.W * g.C, dyimg = (size_t)g.L * g.F;

    int off[G];
#pragma unroll
    for (int gg = 0; gg < G; ++gg) {
        const int k = k0 + gg * 64 + 4 * m;
        const int kc = k < g.K ? k : 0;
        const int kh = kc / g.RC, rem = kc - kh * g.RC;
        off[gg] = ((i * g.S + kh) * g.W + j * g.S) * g.C + rem;
    }
    f32x4 acc[G][4][4];
#pragma unroll
    for (int gg = 0; gg < G; ++gg)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[gg][t][u] = (f32x4){0.f, 0.f, 0.f, 0.f};

    gh_ptr xb = (gh_ptr)x + (size_t)(4 * kk) * img;
    gh_ptr db = (gh_ptr)dy + (size_t)(4 * kk) * dyimg + (size_t)loc * g.F + f0 + 4 * m;
    for (int b0 = 0; b0 < g.B; b0 += 16) {              // B % 16 == 0 on this path
        u32x2 r[4], ao[G][4], bo[4];
#pragma unroll
        for (int gg = 0; gg < G; ++gg) {
#pragma unroll
            for (int t = 0; t < 4; ++t) r[t] = *(g2_ptr)(xb + (size_t)(b0 + t) * img + off[gg]);
            transpose4x4_bf16(r, ao[gg]);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) r[t] = *(g2_ptr)(db + (size_t)(b0 + t) * dyimg);
        transpose4x4_bf16(r, bo);
#pragma unroll
        for (int gg = 0; gg < G; ++gg)
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int u = 0; u < 4; ++u) acc[gg][t][u] = mfma16_bf16(ao[gg][t], bo[u], acc[gg][t][u]);
    }
    float *ol = out + (size_t)loc * g.K * g.F + f0 + 4 * m;
#pragma unroll
    for (int gg = 0; gg < G; ++gg)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int k = k0 + gg * 64 + 4 * (4 * kk + rr) + t;
                if (k >= g.K) continue;
                f32x4 *o = (f32x4 *)(ol + (size_t)k * g.F);
                f32x4 v;
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = acc[gg][t][u][rr];
                if (beta != 0.f) v += beta * *o;
                *o = v;
            }
}

// Shapes this file handles: patch rows, strides and filter counts that keep every 8-byte access aligned.
bool bf16_shape_supported(const Geom &g) {
    return g.RC % 16 == 0 && (g.S * g.C) % 4 == 0 && (g.W * g.C) % 4 == 0 && g.F % 64 == 0 && g.B % 16 == 0 &&
           g.R % g.S == 0;
}

// Order of preference, every pass: the workgroup-tiled kernels (wide layers), the strip-sharing / pipelined / transposing
// kernels of the narrow layers (faster than the one-wave-per-task kernels of this file wherever both apply: the small 32 x 32 x 4 layer
// 30 / 13 / 9 us against 37 / 21 / 10 us), the kernels of this file, the fp32 kernels on bf16 storage.
// Host checks of the one-wave-per-task kernels of this file.  tparam = {MT}; arg as listed per function.
namespace {

// arg = {filter blocks of 64, batch tiles, wave tasks}
int check_forward_bf16_simple(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0], fblocks = p.arg[0], btiles = p.arg[1], ntasks = p.arg[2];
    LC_PLAN_REQUIRE(p, p.block == 256 && bf16_shape_supported(g));
    LC_PLAN_REQUIRE(p, fblocks == g.F / 64 && btiles == ceil_div(g.B, 16 * MT));
    LC_PLAN_REQUIRE(p, (long long)ntasks == (long long)g.L * fblocks * btiles);
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] * 4 >= ntasks && (long long)(p.grid[0] - 1) * 4 < ntasks);
    return LC_OK;
}

// arg = {cells per row, blocks of 64 cell values, batch tiles, wave tasks}
int check_backward_data_bf16_simple(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0], CW = p.arg[0], nblocks = p.arg[1], btiles = p.arg[2], ntasks = p.arg[3];
    LC_PLAN_REQUIRE(p, p.block == 256 && bf16_shape_supported(g));
    LC_PLAN_REQUIRE(p, CW == ceil_div(g.W, g.S) && nblocks == ceil_div(g.S * g.S * g.C, 64) && btiles == ceil_div(g.B, 16 * MT));
    LC_PLAN_REQUIRE(p, (long long)ntasks == (long long)ceil_div(g.H, g.S) * CW * nblocks * btiles);
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] * 4 >= ntasks && (long long)(p.grid[0] - 1) * 4 < ntasks);
    LC_PLAN_REQUIRE(p, (long long)g.K * g.F < (1LL << 31));
    return LC_OK;
}

// arg = {blocks of 128 patch elements per field, wave tasks}
int check_backward_weights_bf16_simple(const Geom &g, const LaunchPlan &p) {
    const int kblocks = p.arg[0], ntasks = p.arg[1];
    LC_PLAN_REQUIRE(p, p.block == 256 && bf16_shape_supported(g));
    LC_PLAN_REQUIRE(p, kblocks == ceil_div(g.K, 128) && (long long)ntasks == (long long)g.L * kblocks);
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] * 4 >= ntasks && (long long)(p.grid[0] - 1) * 4 < ntasks);
    LC_PLAN_REQUIRE(p, (int)p.grid[1] == g.F / 64 && (long long)g.H * g.W * g.C < (1LL << 31));
    return LC_OK;
}

template <int MT>
int launch_forward_simple(const Geom &g, const void *x, const void *w, const float *bias, float alpha, float *y,
                          hipStream_t s) {
    const int fblocks = g.F / 64, btiles = (g.B + 16 * MT - 1) / (16 * MT);
    const long long ntasks = (long long)g.L * fblocks * btiles;
    if (ntasks > (1LL << 30)) return LC_EUNSUPPORTED;
    const LaunchPlan plan = make_plan("lc_forward_bf16_simple", {MT}, {fblocks, btiles, (int)ntasks},
                                      dim3((unsigned)((ntasks + 3) / 4)), 256, 0);
    if (int rc = check_forward_bf16_simple(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_forward (bf16) launch", lc_forward_bf16_kernel<MT>, s, g, (const unsigned short *)x,
              (const unsigned short *)w, bias, alpha, y, fblocks, btiles, (int)ntasks);
    return LC_OK;
}

template <int MT>
int launch_backward_data_simple(const Geom &g, const void *dy, const void *w, float *dx, hipStream_t s) {
    const int CH = (g.H + g.S - 1) / g.S, CW = (g.W + g.S - 1) / g.S;
    const int nblocks = (g.S * g.S * g.C + 63) / 64, btiles = (g.B + 16 * MT - 1) / (16 * MT);
    const long long ntasks = (long long)CH * CW * nblocks * btiles;
    if (ntasks > (1LL << 30)) return LC_EUNSUPPORTED;
    const LaunchPlan plan = make_plan("lc_bwd_data_bf16_simple", {MT}, {CW, nblocks, btiles, (int)ntasks},
                                      dim3((unsigned)((ntasks + 3) / 4)), 256, 0);
    if (int rc = check_backward_data_bf16_simple(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_backward_data (bf16) launch", lc_bwd_data_bf16_kernel<MT>, s, g, (const unsigned short *)dy,
              (const unsigned short *)w, dx, CW, nblocks, btiles, (int)ntasks);
    return LC_OK;
}

}  // namespace

// LC_BF16 covers every valid geometry.  Order of preference, every pass: the workgroup-tiled kernels (wide layers),
// the strip-sharing / pipelined / transposing kernels of the narrow layers (faster than the one-wave-per-task
// kernels of this file wherever both apply), the kernels of this file, the fp32 pipelined kernels on bf16 storage,
// and for every other shape the masked fp32 kernels on bf16 storage.
int launch_forward_bf16(const Geom &g, const void *x, const void *w, const float *bias, float alpha, float *y,
                        hipStream_t s) {
    if (bf16_shape_supported(g) && bf16_tiled_forward_supported(g))
        return launch_forward_bf16_tiled(g, x, w, bias, alpha, y, s);
    if (bf16_strip_forward_supported(g)) return launch_forward_bf16_strip(g, x, w, bias, alpha, y, s);
    if (!bf16_shape_supported(g)) return launch_forward_bf16_storage(g, x, w, bias, alpha, y, s);
    if (g.B >= 64) return launch_forward_simple<4>(g, x, w, bias, alpha, y, s);
    return launch_forward_simple<1>(g, x, w, bias, alpha, y, s);
}

int launch_backward_data_bf16(const Geom &g, const void *dy, const void *w, float *dx, hipStream_t s) {
    if (bf16_shape_supported(g) && bf16_tiled_backward_data_supported(g))
        return launch_backward_data_bf16_tiled(g, dy, w, dx, s);
    if (!bf16_shape_supported(g) || backward_data_bf16_pipelined_supported(g))
        return launch_backward_data_bf16_storage(g, dy, w, dx, s);   // pipelined (bf16 MFMAs) or masked kernel
    if (g.B >= 128) return launch_backward_data_simple<8>(g, dy, w, dx, s);
    if (g.B >= 64) return launch_backward_data_simple<4>(g, dy, w, dx, s);
    return launch_backward_data_simple<1>(g, dy, w, dx, s);
}

int launch_backward_weights_bf16(const Geom &g, const void *x, const void *dy, float beta, float *dw,
                                 hipStream_t s) {
    if (bf16_shape_supported(g) && bf16_tiled_backward_weights_supported(g))
        return launch_backward_weights_bf16_tiled(g, x, dy, beta, dw, s);
    if (bf16_rows_backward_weights_supported(g)) return launch_backward_weights_bf16_rows(g, x, dy, beta, dw, s);
    if (!bf16_shape_supported(g)) return launch_backward_weights_bf16_storage(g, x, dy, beta, dw, s);
    const int kblocks = (g.K + 127) / 128;
    const long long ntasks = (long long)g.L * kblocks;
    if (ntasks > (1LL << 30)) return LC_EUNSUPPORTED;
    const LaunchPlan plan = make_plan("lc_bwd_weights_bf16_simple", {}, {kblocks, (int)ntasks},
                                      dim3((unsigned)((ntasks + 3) / 4), g.F / 64), 256, 0);
    if (int rc = check_backward_weights_bf16_simple(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_backward_weights (bf16) launch", lc_bwd_weights_bf16_kernel, s, g, (const unsigned short *)x,
              (const unsigned short *)dy, beta, dw, kblocks, (int)ntasks);
    return LC_OK;
}

}  // namespace lc
