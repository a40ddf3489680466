// lc_forward: y[b,l,f] = alpha * sum_k w[l,k,f] * patch(x)[b,l,k] + bias[l,f]   (Eq. 1's "alpha W x",
// untied receptive fields of Sec. 3.1).
//
// One workgroup (4 waves) owns a run of NLOC horizontally adjacent locations of one location row, a
// batch tile of BT = 16*MT images and 4/NLOC blocks of 16*NT filters.  Adjacent fields overlap by
// R-S pixels, so the workgroup stages one image-row strip covering all its fields in LDS (coalesced
// reads along the contiguous (w,c) run of an [H][W][C] image) and every wave reads its own window
// of it.  A wave holds the whole batch tile for its location: each weight is fetched from global
// memory exactly once per batch tile, straight into the MFMA B operand (lanes run along f, the
// contiguous axis of w), and reused for MT MFMAs.
#include "lc_common.hpp"

namespace lc {

template <int MT, int NT, int NLOC, bool MASK>
__device__ __forceinline__ void fwd_row(f32x4 (&acc)[MT][NT], const float *__restrict__ xs_win, int rs,
                                        const float *__restrict__ wrow, int F, int RC, int kk, bool (&fok)[NT]) {
    const int lane_m = threadIdx.x & 15;
#pragma unroll 2
    for (int kq = 0; kq < RC; kq += 4) {
        float bw[NT], a[MT];
        const bool kok = !MASK || (kq + kk < RC);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (MASK)
                bw[nt] = (kok && fok[nt]) ? wrow[(size_t)kq * F + nt * 16] : 0.f;
            else
                bw[nt] = wrow[(size_t)kq * F + nt * 16];
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const float v = xs_win[(mt * 16 + lane_m) * rs + kq];
            a[mt] = (!MASK || kok) ? v : 0.f;
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = mfma16(a[mt], bw[nt], acc[mt][nt]);
    }
}

template <int MT, int NT, int NLOC>
__global__ __launch_bounds__(256) void lc_forward_kernel(Geom g, const float *__restrict__ x,
                                                         const float *__restrict__ w,
                                                         const float *__restrict__ bias, float alpha,
                                                         const float *__restrict__ alpha_dev,
                                                         float *__restrict__ y, int strips_per_row, int sq, int rs) {
    constexpr int BT = 16 * MT, NFW = 4 / NLOC;
    extern __shared__ float xs[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, kk = lane >> 4;
    const int work = remap_xcd(blockIdx.x, gridDim.x);
    const int i = work / strips_per_row, j0 = (work - i * strips_per_row) * NLOC;
    const int b0 = blockIdx.z * BT;
    const int wl = wave % NLOC, wf = wave / NLOC;
    const int j = j0 + wl;
    const int f0 = (blockIdx.y * NFW + wf) * NT * 16;
    const bool active = (j < g.LW) && (f0 < g.F);
    const int loc = i * g.LW + (active ? j : 0);

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

    bool fok[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) fok[nt] = active && (f0 + nt * 16 + n < g.F);
    const bool need_mask = (g.RC & 3) != 0 || (f0 + NT * 16 > g.F);

    // strip staging: thread t copies elements t, t+256, ... of the [BT][sq] strip (q fastest)
    const int q_first = tid % sq, b_first = tid / sq, dq = 256 % sq, db = 256 / sq;
    const int col0 = j0 * g.S * g.C;                       // first float of the strip inside an image row
    const int nvalid = min(sq, g.W * g.C - col0);          // strip floats that exist in the image
    const size_t img = (size_t)g.H * g.W * g.C;
    const float *wl_base = w + (size_t)loc * g.K * g.F + f0 + n;
    const float *xs_win = xs + wl * g.S * g.C + kk;

    for (int kh = 0; kh < g.R; ++kh) {
        __syncthreads();
        {
            const float *xrow = x + (size_t)(i * g.S + kh) * g.W * g.C + col0;
            int q = q_first, bb = b_first;
            while (bb < BT) {
                float v = 0.f;
                if (q < nvalid && b0 + bb < g.B) v = xrow[(size_t)(b0 + bb) * img + q];
                xs[bb * rs + q] = v;
                q += dq;
                bb += db;
                if (q >= sq) { q -= sq; ++bb; }
            }
        }
        __syncthreads();
        if (active) {
            const float *wrow = wl_base + (size_t)(kh * g.RC + kk) * g.F;
            if (need_mask)
                fwd_row<MT, NT, NLOC, true>(acc, xs_win, rs, wrow, g.F, g.RC, kk, fok);
            else
                fwd_row<MT, NT, NLOC, false>(acc, xs_win, rs, wrow, g.F, g.RC, kk, fok);
        }
    }

    if (!active) return;
    if (alpha_dev) alpha = *alpha_dev;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int f = f0 + nt * 16 + n;
        if (f >= g.F) continue;
        const float bv = bias ? bias[(size_t)loc * g.F + f] : 0.f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int b = b0 + mt * 16 + 4 * kk + r;
                if (b < g.B) y[((size_t)b * g.L + loc) * g.F + f] = alpha * acc[mt][nt][r] + bv;
            }
    }
}

namespace {

struct FwdPlan { int MT, NT, NLOC; };

// LDS budget per workgroup: at most 64 KB so that two workgroups share a compute unit's 160 KB.
constexpr size_t kLdsTarget = 64 * 1024;

int lds_row_stride(int sq) {
    // row stride == 2 (mod 32): the 16 image rows a wave reads at once fall into distinct LDS banks
    int rs = ((sq + 3 + 31) / 32) * 32 + 2;
    if (rs - 32 >= sq + 3) rs -= 32;
    return rs;
}

template <int MT, int NT, int NLOC>
int launch_one(const Geom &g, const float *x, const float *w, const float *bias, float alpha,
               const float *alpha_dev, float *y, hipStream_t s) {
    constexpr int BT = 16 * MT, NFW = 4 / NLOC;
    const int strips = (g.LW + NLOC - 1) / NLOC;
    const int sq = (g.R + (NLOC - 1) * g.S) * g.C;
    const int rs = lds_row_stride(sq);
    const size_t lds = ((size_t)BT * rs + 8) * sizeof(float);
    if (lds > 160 * 1024) return LC_EUNSUPPORTED;
    auto kern = lc_forward_kernel<MT, NT, NLOC>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { set_hip_error(e, "lc_forward: hipFuncSetAttribute"); return LC_EHIP; }
    }
    dim3 grid(strips * g.LH, (g.F + NFW * NT * 16 - 1) / (NFW * NT * 16), (g.B + BT - 1) / BT);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, g, x, w, bias, alpha, alpha_dev, y, strips, sq, rs);
    LC_HIP_LAUNCH_CHECK("lc_forward launch");
    return LC_OK;
}

}  // namespace

int launch_forward_f32(const Geom &g, const float *x, const float *w, const float *bias, float alpha,
                       const float *alpha_dev, float *y, hipStream_t s) {
    // Pick the tile: as many images per wave as the batch offers (weights are re-read once per batch
    // tile), then as many filters as fit the accumulator budget, then the widest strip that fits LDS.
    const int mt = g.B > 64 ? 8 : g.B > 32 ? 4 : g.B > 16 ? 2 : 1;
    const int ft = (g.F + 15) / 16;  // filter tiles
    auto strip_bytes = [&](int nloc, int MT) {
        return ((size_t)16 * MT * lds_row_stride((g.R + (nloc - 1) * g.S) * g.C) + 8) * sizeof(float);
    };
#define LC_TRY(MT_, NT_, NLOC_) return launch_one<MT_, NT_, NLOC_>(g, x, w, bias, alpha, alpha_dev, y, s)
    if (mt == 8) {
        if (ft <= 2 && strip_bytes(4, 8) <= kLdsTarget) { if (ft == 1) LC_TRY(8, 1, 4); LC_TRY(8, 2, 4); }
        if (ft <= 4 && strip_bytes(2, 8) <= kLdsTarget) LC_TRY(8, 2, 2);
        if (strip_bytes(1, 8) <= 2 * kLdsTarget) LC_TRY(8, 2, 1);
        if (strip_bytes(2, 4) <= kLdsTarget) LC_TRY(4, 4, 2);
        if (strip_bytes(1, 4) <= 2 * kLdsTarget) LC_TRY(4, 4, 1);
        if (strip_bytes(1, 2) <= 2 * kLdsTarget) LC_TRY(2, 4, 1);
        LC_TRY(1, 4, 1);
    }
    if (mt == 4) {
        if (ft <= 2 && strip_bytes(4, 4) <= kLdsTarget) LC_TRY(4, 2, 4);
        if (strip_bytes(2, 4) <= kLdsTarget) LC_TRY(4, 4, 2);
        if (strip_bytes(1, 4) <= 2 * kLdsTarget) LC_TRY(4, 4, 1);
        if (strip_bytes(1, 2) <= 2 * kLdsTarget) LC_TRY(2, 4, 1);
        LC_TRY(1, 4, 1);
    }
    if (mt == 2) {
        if (ft <= 2 && strip_bytes(4, 2) <= kLdsTarget) LC_TRY(2, 2, 4);
        if (strip_bytes(1, 2) <= 2 * kLdsTarget) LC_TRY(2, 4, 1);
        LC_TRY(1, 4, 1);
    }
    if (ft <= 2 && strip_bytes(4, 1) <= kLdsTarget) LC_TRY(1, 2, 4);
    LC_TRY(1, 4, 1);
#undef LC_TRY
}

}  // namespace lc
