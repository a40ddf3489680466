// lc_backward_weights: out[l,k,f] = beta*out[l,k,f] + gamma * sum_p sum_b patch(x_p)[b,l,k] * dy_p[b,l,f]
// (the weight gradient of Eq. 1; two operand pairs because the tied weights are used twice).
//
// The contraction runs over the batch, so both MFMA operands are read straight from global memory
// with lanes along the contiguous axis: A[k][b] lanes run along k (the (kw,c) run of an image row),
// B[b][f] lanes run along f.  Waves are independent: each owns one location, MTW tiles of 16 patch
// elements and NT tiles of 16 filters, loops over the batch four images at a time and writes its
// MTW x NT output tiles once.
#include "lc_common.hpp"

namespace lc {

template <int MTW, int NT>
__global__ __launch_bounds__(256) void lc_bwd_weights_kernel(Geom g, const float *__restrict__ x1,
                                                             const float *__restrict__ dy1,
                                                             const float *__restrict__ x2,
                                                             const float *__restrict__ dy2, float beta, float gamma,
                                                             float *__restrict__ out, int kblocks, int ntasks) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, kk = lane >> 4;
    const int task = remap_xcd(blockIdx.x, gridDim.x) * 4 + wave;
    if (task >= ntasks) return;
    const int loc = task / kblocks, k0 = (task - loc * kblocks) * MTW * 16;
    const int i = loc / g.LW, j = loc - i * g.LW;
    const int f0 = blockIdx.y * NT * 16;
    const size_t img = (size_t)g.H * g.W * g.C;

    int off[MTW];
    bool kok[MTW];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        const int k = k0 + mt * 16 + m;
        kok[mt] = k < g.K;
        const int kc = kok[mt] ? k : 0;
        const int kh = kc / g.RC, rem = kc - kh * g.RC;
        off[mt] = ((i * g.S + kh) * g.W + j * g.S) * g.C + rem;
    }
    bool fok[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) fok[nt] = f0 + nt * 16 + m < g.F;

    f32x4 acc[MTW][NT];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int Bfull = g.B & ~3;
    const bool edge = (k0 + MTW * 16 > g.K) || (f0 + NT * 16 > g.F);
    for (int p = 0; p < 2; ++p) {
        const float *x = p ? x2 : x1;
        const float *dy = p ? dy2 : dy1;
        if (!x) break;
        const float *xa = x + (size_t)kk * img;
        const float *da = dy + ((size_t)kk * g.L + loc) * g.F + f0 + m;
        const size_t dstep = (size_t)g.L * g.F;
        if (!edge) {
#pragma unroll 2
            for (int b0 = 0; b0 < Bfull; b0 += 4) {
                float a[MTW], bv[NT];
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt) a[mt] = xa[(size_t)b0 * img + off[mt]];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) bv[nt] = da[(size_t)b0 * dstep + nt * 16];
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = mfma16(a[mt], bv[nt], acc[mt][nt]);
            }
        }
        // ragged tiles, and the last 1-3 images of a batch that is not a multiple of 4
        for (int b0 = edge ? 0 : Bfull; b0 < g.B; b0 += 4) {
            const bool bok = b0 + kk < g.B;
            float a[MTW], bv[NT];
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) a[mt] = (bok && kok[mt]) ? xa[(size_t)b0 * img + off[mt]] : 0.f;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) bv[nt] = (bok && fok[nt]) ? da[(size_t)b0 * dstep + nt * 16] : 0.f;
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = mfma16(a[mt], bv[nt], acc[mt][nt]);
        }
    }

    float *ol = out + (size_t)loc * g.K * g.F;
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int k = k0 + mt * 16 + 4 * kk + r;
            if (k >= g.K) continue;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                if (!fok[nt]) continue;
                float *o = ol + (size_t)k * g.F + f0 + nt * 16 + m;
                const float v = gamma * acc[mt][nt][r];
                *o = (beta != 0.f) ? beta * *o + v : v;
            }
        }
}

namespace {

template <int MTW, int NT>
int launch_one(const Geom &g, const float *x1, const float *dy1, const float *x2, const float *dy2, float beta,
               float gamma, float *out, hipStream_t s) {
    const int kt = (g.K + 15) / 16;
    const int kblocks = (kt + MTW - 1) / MTW;
    const long long ntasks = (long long)g.L * kblocks;
    if (ntasks > (1LL << 30)) return LC_EUNSUPPORTED;
    dim3 grid((unsigned)((ntasks + 3) / 4), (g.F + NT * 16 - 1) / (NT * 16));
    hipLaunchKernelGGL((lc_bwd_weights_kernel<MTW, NT>), grid, dim3(256), 0, s, g, x1, dy1, x2, dy2, beta, gamma,
                       out, kblocks, (int)ntasks);
    LC_HIP_LAUNCH_CHECK("lc_backward_weights launch");
    return LC_OK;
}

template <int NT>
int launch_nt(const Geom &g, const float *x1, const float *dy1, const float *x2, const float *dy2, float beta,
              float gamma, float *out, hipStream_t s) {
    // tiles of 16 patch elements per wave: the candidate with the least padding of K, larger first
    const int kt = (g.K + 15) / 16;
    const int cand[4] = {8, 6, 5, 4};
    int best = 8, waste = 1 << 30;
    for (int c : cand) {
        const int wst = (kt + c - 1) / c * c - kt;
        if (wst < waste) { waste = wst; best = c; }
    }
    switch (best) {
        case 8: return launch_one<8, NT>(g, x1, dy1, x2, dy2, beta, gamma, out, s);
        case 6: return launch_one<6, NT>(g, x1, dy1, x2, dy2, beta, gamma, out, s);
        case 5: return launch_one<5, NT>(g, x1, dy1, x2, dy2, beta, gamma, out, s);
        default: return launch_one<4, NT>(g, x1, dy1, x2, dy2, beta, gamma, out, s);
    }
}

}  // namespace

int launch_backward_weights_f32(const Geom &g, const float *x1, const float *dy1, const float *x2, const float *dy2,
                                float beta, float gamma, float *out, hipStream_t s) {
    if (g.F <= 16) return launch_nt<1>(g, x1, dy1, x2, dy2, beta, gamma, out, s);
    if (g.F <= 32) return launch_nt<2>(g, x1, dy1, x2, dy2, beta, gamma, out, s);
    return launch_nt<4>(g, x1, dy1, x2, dy2, beta, gamma, out, s);
}

}  // namespace lc
