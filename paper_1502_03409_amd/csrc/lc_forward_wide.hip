// lc_forward for wide layers (F a multiple of 128, patch rows that split into chunks of 32 values): Eq. 1's
// encoder term with a workgroup tile of one field x 128 filters x 32*MT images.
//
// The four waves form a 2 x 2 grid (16*MT images x 64 filters each).  The field's patch rows reach the waves
// through LDS in chunks of 32 contraction indices (128 contiguous bytes per image, two buffers, one barrier per
// chunk); both image halves of a filter half load the same weights at the same time, so the CU's vector cache
// serves the second.  A chunk is two groups of 16 indices: lane (m, kk) reads indices 4kk..4kk+3 of a group as
// one 16-byte LDS read and uses component t in MFMA step t, and lane (n, kk) loads the weight rows 4kk+t at
// filters 4n..4n+3 (16 lanes cover 256 contiguous bytes), which makes column n of filter tile u filter 4n+u.
#include "lc_common.hpp"

namespace lc {

namespace {

typedef const __attribute__((address_space(1))) f32x4 *g4_ptr;
typedef const __attribute__((address_space(1))) float *gf_ptr;

constexpr int kChunk = 32;          // contraction indices per LDS chunk
constexpr int kRowFloats = 36;      // 32 floats of a chunk + 4: eight rows' 16-byte reads cover all banks

template <int MT, int PD>
__global__ __launch_bounds__(256, 2) void lc_forward_wide_kernel(Geom g, const float *__restrict__ x,
                                                                 const float *__restrict__ w,
                                                                 const float *__restrict__ bias, float alpha,
                                                                 const float *__restrict__ alpha_dev,
                                                                 float *__restrict__ y, int fblocks, int btiles) {
    static_assert(PD == 1 || PD == 2, "one or two chunks of lookahead");
    constexpr int BT = 32 * MT, NS = MT;          // NS: 16-byte staging slots per thread and chunk
    constexpr int BUF = BT * kRowFloats;
    extern __shared__ __attribute__((aligned(16))) float xs[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, kk = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    // batch tiles of one (field, filter block) are neighbours in dispatch order: they share the filters in L2
    int t_id = remap_xcd(blockIdx.x, gridDim.x);
    const int bt = t_id % btiles;
    t_id /= btiles;
    const int fb = t_id % fblocks, loc = t_id / fblocks;
    const int i = loc / g.LW, j = loc - i * g.LW;
    const int b0 = bt * BT, f0 = fb * 128 + wn * 64;
    const int WC = g.W * g.C;
    const int cpr = g.RC / kChunk, nchunks = g.R * cpr;

    f32x4 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[mt][u] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // staging: slot s moves 16 bytes (segment tid&7) of image (tid>>3) + 32 s; images beyond the batch
    // repeat image B-1 and their results are never stored
    const int seg = tid & 7, brow = tid >> 3;
    int xoff[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int b = min(b0 + brow + 32 * s, g.B - 1);
        xoff[s] = (b * g.H + i * g.S) * WC + j * g.S * g.C + seg * 4;
    }
    auto stage_load = [&](int c, f32x4 (&st)[NS]) {
        const int kh = c / cpr;
        const int o = kh * WC + (c - kh * cpr) * kChunk;
#pragma unroll
        for (int s = 0; s < NS; ++s) st[s] = *(g4_ptr)((gf_ptr)x + xoff[s] + o);
    };
    auto stage_store = [&](int buf, const f32x4 (&st)[NS]) {
#pragma unroll
        for (int s = 0; s < NS; ++s) *(f32x4 *)(xs + buf * BUF + (brow + 32 * s) * kRowFloats + seg * 4) = st[s];
    };
    // filters: the chunks tile k contiguously; group q covers rows 16q .. 16q+15 of the field's K x F matrix
    gf_ptr wl = (gf_ptr)w + (size_t)loc * g.K * g.F + f0 + 4 * n + (size_t)(4 * kk) * g.F;
    const int ngroups = 2 * nchunks;
    auto wload = [&](int q, f32x4 (&r)[4]) {
        gf_ptr p = wl + (size_t)(16 * min(q, ngroups - 1)) * g.F;
#pragma unroll
        for (int t = 0; t < 4; ++t) r[t] = *(g4_ptr)(p + t * g.F);
    };

    f32x4 st[PD][NS];
    f32x4 wr[2 * PD][4];
#pragma unroll
    for (int q = 0; q < 2 * PD; ++q) wload(q, wr[q]);
    stage_load(0, st[0]);
    stage_store(0, st[0]);
#pragma unroll
    for (int p = 0; p < PD; ++p) stage_load(min(p + 1, nchunks - 1), st[p]);      // set p: chunk p+1
    __syncthreads();
    const int arow = (wm * 16 * MT + n) * kRowFloats + 4 * kk;
    for (int c0 = 0; c0 < nchunks; c0 += 2) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int c = c0 + p;               // chunk c lives in buffer p (c0 is even)
            const int sp = p % PD;              // register set that holds chunk c+1
            if (c < nchunks) {
                const float *ab = xs + p * BUF + arow;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    f32x4 bo[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) bo[t] = wr[2 * sp + h][t];
                    wload(2 * c + h + 2 * PD, wr[2 * sp + h]);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const f32x4 a = *(const f32x4 *)(ab + mt * 16 * kRowFloats + 16 * h);
#pragma unroll
                        for (int t = 0; t < 4; ++t)
#pragma unroll
                            for (int u = 0; u < 4; ++u) acc[mt][u] = mfma16(a[t], bo[t][u], acc[mt][u]);
                    }
                }
                // the other buffer was last read in chunk c-1, which every wave left at the previous barrier
                if (c + 1 < nchunks) stage_store(p ^ 1, st[sp]);
                if (c + 1 + PD < nchunks) stage_load(c + 1 + PD, st[sp]);
            }
            __syncthreads();
        }
    }

    if (alpha_dev) alpha = *alpha_dev;
    f32x4 bv = (f32x4){0.f, 0.f, 0.f, 0.f};
    if (bias) bv = *(const f32x4 *)(bias + (size_t)loc * g.F + f0 + 4 * n);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int b = b0 + wm * 16 * MT + mt * 16 + 4 * kk + rr;
            if (b >= g.B) continue;
            f32x4 o;
#pragma unroll
            for (int u = 0; u < 4; ++u) o[u] = alpha * acc[mt][u][rr] + bv[u];
            *(f32x4 *)(y + ((size_t)b * g.L + loc) * g.F + f0 + 4 * n) = o;
        }
}

template <int MT, int PD>
int launch_wide(const Geom &g, const float *x, const float *w, const float *bias, float alpha, const float *alpha_dev,
                float *y, hipStream_t s) {
    constexpr int BT = 32 * MT;
    const size_t lds = (size_t)2 * BT * kRowFloats * sizeof(float);
    auto kern = lc_forward_wide_kernel<MT, PD>;
    if (int rc_lds = allow_dynamic_lds((const void *)kern, lds, "lc_forward (wide): hipFuncSetAttribute")) return rc_lds;
    const int fblocks = g.F / 128, btiles = (g.B + BT - 1) / BT;
    hipLaunchKernelGGL(kern, dim3((unsigned)(g.L * fblocks * btiles)), dim3(256), lds, s, g, x, w, bias, alpha,
                       alpha_dev, y, fblocks, btiles);
    LC_HIP_LAUNCH_CHECK("lc_forward (wide) launch");
    return LC_OK;
}

}  // namespace

bool forward_wide_supported(const Geom &g) {
    return g.F % 128 == 0 && g.RC % kChunk == 0 && (g.S * g.C) % 4 == 0 && (g.W * g.C) % 4 == 0 && g.B > 64 &&
           (long long)g.B * g.H * g.W * g.C < (1ll << 31) &&
           (long long)g.L * (g.F / 128) * ((g.B + 127) / 128) < (1ll << 31);
}

int launch_forward_wide_f32(const Geom &g, const float *x, const float *w, const float *bias, float alpha,
                            const float *alpha_dev, float *y, hipStream_t s) {
    if (!forward_wide_supported(g)) return LC_EUNSUPPORTED;
    // 128-image tiles measured faster than 256-image ones here (1062 vs 1116 us on 256 x 64x64x32, 128 filters)
    return launch_wide<4, 2>(g, x, w, bias, alpha, alpha_dev, y, s);
}

}  // namespace lc
