// lc_forward for wide layers (F a multiple of 128, patch rows that split into chunks of 32 or 16 values): Eq. 1's
// encoder term with a workgroup tile of one field x 128 filters x 32*MT images.
//
// The four waves form a 2 x 2 grid (16*MT images x 64 filters each).  The field's patch rows reach the waves
// through LDS in chunks of 32 contraction indices (128 contiguous bytes per image, two buffers, one barrier per
// chunk); both image halves of a filter half load the same weights at the same time, so the CU's vector cache
// serves the second.  A chunk is two groups of 16 indices: lane (m, kk) reads indices 4kk..4kk+3 of a group as
// one 16-byte LDS read and uses component t in MFMA step t, and lane (n, kk) loads the weight rows 4kk+t at
// filters 4n..4n+3 (16 lanes cover 256 contiguous bytes), which makes column n of filter tile u filter 4n+u.
#include <algorithm>

#include "lc_common.hpp"

namespace lc {

namespace {

typedef const __attribute__((address_space(1))) f32x4 *g4_ptr;
typedef const __attribute__((address_space(1))) float *gf_ptr;

// KCH = contraction indices per LDS chunk (32, or 16 for patch rows that are only a multiple of 16): KCH*4
// contiguous bytes per image, rows padded by 16 bytes so that eight rows' 16-byte reads cover all banks.
//
// A layer with few fields (the dense last layer of Sec. 3.1 is a single one) gives too few workgroups; its
// contraction is then cut into `nslices` ranges of chunks, each range a workgroup of its own that writes a partial
// result into the caller's workspace, and a second kernel adds the slices in a fixed order and applies alpha and
// the bias.
template <int MT, int PD, int KCH>
__global__ __launch_bounds__(256, 2) void lc_forward_wide_kernel(Geom g, const float *__restrict__ x,
                                                                 const float *__restrict__ w,
                                                                 const float *__restrict__ bias, float alpha,
                                                                 const float *__restrict__ alpha_dev,
                                                                 float *__restrict__ y, float *__restrict__ partial,
                                                                 int fblocks, int btiles, int nslices) {
    static_assert(PD == 1 || PD == 2, "one or two chunks of lookahead");
    constexpr int ROWF = KCH + 4, SEGS = KCH / 4, SR = 256 / SEGS, GPC = KCH / 16;
    constexpr int BT = 32 * MT, NS = BT / SR;     // NS: 16-byte staging slots per thread and chunk
    constexpr int BUF = BT * ROWF;
    static_assert(NS >= 1, "batch tile too small for the staging map");
    extern __shared__ __attribute__((aligned(16))) float xs[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, kk = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    // batch tiles of one (field, filter block) are neighbours in dispatch order: they share the filters in L2
    int t_id = remap_xcd(blockIdx.x, gridDim.x);
    const int bt = t_id % btiles;
    t_id /= btiles;
    const int fb = t_id % fblocks;
    t_id /= fblocks;
    const int loc = t_id % g.L, slice = t_id / g.L;
    const int i = loc / g.LW, j = loc - i * g.LW;
    const int b0 = bt * BT, f0 = fb * 128 + wn * 64;
    const int WC = g.W * g.C;
    const int cpr = g.RC / KCH, nchunks_all = g.R * cpr;
    // this workgroup's range of chunks
    const int c_lo = (int)((long long)nchunks_all * slice / nslices);
    const int c_hi = (int)((long long)nchunks_all * (slice + 1) / nslices);
    const int nchunks = c_hi - c_lo;

    f32x4 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[mt][u] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // staging: slot s moves 16 bytes (segment tid % SEGS) of image tid / SEGS + SR s; images beyond the batch
    // repeat image B-1 and their results are never stored
    const int seg = tid % SEGS, brow = tid / SEGS;
    int xoff[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int b = min(b0 + brow + SR * s, g.B - 1);
        xoff[s] = (b * g.H + i * g.S) * WC + j * g.S * g.C + seg * 4;
    }
    auto stage_load = [&](int c, f32x4 (&st)[NS]) {          // c: chunk index relative to c_lo
        const int ca = c_lo + min(c, nchunks - 1), kh = ca / cpr;
        const int o = kh * WC + (ca - kh * cpr) * KCH;
#pragma unroll
        for (int s = 0; s < NS; ++s) st[s] = *(g4_ptr)((gf_ptr)x + xoff[s] + o);
    };
    auto stage_store = [&](int buf, const f32x4 (&st)[NS]) {
#pragma unroll
        for (int s = 0; s < NS; ++s) *(f32x4 *)(xs + buf * BUF + (brow + SR * s) * ROWF + seg * 4) = st[s];
    };
    // filters: the chunks tile k contiguously; group q covers rows 16q .. 16q+15 of the field's K x F matrix
    gf_ptr wl = (gf_ptr)w + (size_t)loc * g.K * g.F + f0 + 4 * n + (size_t)(4 * kk) * g.F;
    const int q_lo = c_lo * GPC, ngroups = nchunks * GPC;
    auto wload = [&](int q, f32x4 (&r)[4]) {                // q: group index relative to q_lo
        gf_ptr p = wl + (size_t)(16 * (q_lo + min(q, ngroups - 1))) * g.F;
#pragma unroll
        for (int t = 0; t < 4; ++t) r[t] = *(g4_ptr)(p + t * g.F);
    };

    if (nchunks > 0) {
        f32x4 st[PD][NS];
        f32x4 wr[GPC * PD][4];
#pragma unroll
        for (int q = 0; q < GPC * PD; ++q) wload(q, wr[q]);
        stage_load(0, st[0]);
        stage_store(0, st[0]);
#pragma unroll
        for (int p = 0; p < PD; ++p) stage_load(p + 1, st[p]);      // set p: chunk p+1
        __syncthreads();
        const int arow = (wm * 16 * MT + n) * ROWF + 4 * kk;
        for (int c0 = 0; c0 < nchunks; c0 += 2) {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int c = c0 + p;               // chunk c lives in buffer p (c0 is even)
                const int sp = p % PD;              // register set that holds chunk c+1
                if (c < nchunks) {
                    const float *ab = xs + p * BUF + arow;
#pragma unroll
                    for (int h = 0; h < GPC; ++h) {
                        f32x4 bo[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) bo[t] = wr[GPC * sp + h][t];
                        wload(GPC * c + h + GPC * PD, wr[GPC * sp + h]);
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            const f32x4 a = *(const f32x4 *)(ab + mt * 16 * ROWF + 16 * h);
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
    }

    const bool whole = nslices == 1;
    if (whole && alpha_dev) alpha = *alpha_dev;
    f32x4 bv = (f32x4){0.f, 0.f, 0.f, 0.f};
    if (whole && bias) bv = *(const f32x4 *)(bias + (size_t)loc * g.F + f0 + 4 * n);
    float *yo = whole ? y : partial + (size_t)slice * g.B * g.L * g.F;
    const float sc = whole ? alpha : 1.f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int b = b0 + wm * 16 * MT + mt * 16 + 4 * kk + rr;
            if (b >= g.B) continue;
            f32x4 o;
#pragma unroll
            for (int u = 0; u < 4; ++u) o[u] = sc * acc[mt][u][rr] + bv[u];
            *(f32x4 *)(yo + ((size_t)b * g.L + loc) * g.F + f0 + 4 * n) = o;
        }
}

// y = alpha * (sum of the slices, in order) + bias
__global__ __launch_bounds__(256) void lc_forward_slices_kernel(const float *__restrict__ partial, int nslices,
                                                                size_t n4, int LF4, const float *__restrict__ bias,
                                                                float alpha, const float *__restrict__ alpha_dev,
                                                                float *__restrict__ y) {
    if (alpha_dev) alpha = *alpha_dev;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n4; e += (size_t)gridDim.x * 256) {
        f32x4 s = ((const f32x4 *)partial)[e];
        for (int k = 1; k < nslices; ++k) s += ((const f32x4 *)partial)[(size_t)k * n4 + e];
        f32x4 bv = (f32x4){0.f, 0.f, 0.f, 0.f};
        if (bias) bv = ((const f32x4 *)bias)[e % (size_t)LF4];
        ((f32x4 *)y)[e] = alpha * s + bv;
    }
}

int chunk_floats(const Geom &g) { return g.RC % 32 == 0 ? 32 : 16; }

// slices that would give a layer with few fields about two rounds of workgroups; 1 = no split
int wide_slices(const Geom &g) {
    const long long wgs = (long long)g.L * (g.F / 128) * ((g.B + 127) / 128);
    if (wgs >= 256) return 1;
    const int nchunks = g.R * (g.RC / chunk_floats(g));
    int ns = (int)((1024 + wgs - 1) / wgs);
    if (ns > 16) ns = 16;
    if (ns > nchunks / 8) ns = nchunks / 8;      // keep slices long enough to amortise their pipeline fill
    return ns < 2 ? 1 : ns;
}

// Host check of a lc_forward_wide_kernel launch.  tparam = {MT, PD, KCH}; arg = {filter blocks, batch tiles, slices}.
int check_forward_wide(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0], KCH = p.tparam[2];
    const int fblocks = p.arg[0], btiles = p.arg[1], nslices = p.arg[2];
    const int BT = 32 * MT, SEGS = KCH / 4, SR = 256 / SEGS;
    LC_PLAN_REQUIRE(p, p.block == 256 && (KCH == 32 || KCH == 16));
    // 128 filters per workgroup; patch rows in whole chunks whose starts are 16-byte aligned in every image row
    LC_PLAN_REQUIRE(p, g.F % 128 == 0 && fblocks == g.F / 128);
    LC_PLAN_REQUIRE(p, g.RC % KCH == 0 && (g.S * g.C) % 4 == 0 && (g.W * g.C) % 4 == 0);
    // the staging map: 256 threads move SR image rows per slot, BT / SR whole slots
    LC_PLAN_REQUIRE(p, BT % SR == 0 && BT / SR >= 1);
    LC_PLAN_REQUIRE(p, btiles == ceil_div(g.B, BT));
    // 32-bit element offsets of x
    LC_PLAN_REQUIRE(p, (long long)g.B * g.H * g.W * g.C < (1LL << 31));
    const int nchunks = g.R * (g.RC / KCH);
    LC_PLAN_REQUIRE(p, nslices >= 1 && nslices <= nchunks);
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] == (long long)g.L * fblocks * btiles * nslices && p.grid[1] == 1 &&
                           p.grid[2] == 1);
    LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)2 * BT * (KCH + 4) * sizeof(float));
    return LC_OK;
}

template <int KCH, int MT = 4>
int launch_wide(const Geom &g, const float *x, const float *w, const float *bias, float alpha, const float *alpha_dev,
                float *y, float *partial, int nslices, hipStream_t s) {
    constexpr int PD = 2, BT = 32 * MT;
    const size_t lds = (size_t)2 * BT * (KCH + 4) * sizeof(float);
    auto kern = lc_forward_wide_kernel<MT, PD, KCH>;
    const int fblocks = g.F / 128, btiles = (g.B + BT - 1) / BT;
    const LaunchPlan plan = make_plan("lc_forward_wide", {MT, PD, KCH}, {fblocks, btiles, nslices},
                                      dim3((unsigned)(g.L * fblocks * btiles * nslices)), 256, lds);
    if (int rc = check_forward_wide(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_forward (wide) launch", kern, s, g, x, w, bias, alpha, alpha_dev, y, partial, fblocks, btiles,
              nslices);
    if (nslices > 1) {
        const size_t n4 = (size_t)g.B * g.L * g.F / 4;
        const unsigned blocks = (unsigned)std::min<size_t>((n4 + 255) / 256, 256 * 16);
        const LaunchPlan sum = make_plan("lc_forward_slices", {}, {nslices}, dim3(blocks), 256, 0);
        LC_LAUNCH(sum, "lc_forward (slices) launch", lc_forward_slices_kernel, s, partial, nslices, n4, g.L * g.F / 4,
                  bias, alpha, alpha_dev, y);
    }
    return LC_OK;
}

}  // namespace

// 128-filter blocks, patch rows that split into chunks with 16-byte aligned starts, offsets in 32 bits.  Chunks of
// 32 values always; chunks of 16 only for layers with few fields: with many overlapping fields of few channels
// (the paper's first layer) the strip-sharing kernel reads the patches far less often and is the faster one.
bool forward_wide_supported(const Geom &g) {
    const bool few_fields = (long long)g.L * (g.F / 128) * ((g.B + 127) / 128) < 256;
    return g.F % 128 == 0 && (g.RC % 32 == 0 || (g.RC % 16 == 0 && few_fields)) && (g.S * g.C) % 4 == 0 &&
           (g.W * g.C) % 4 == 0 && g.B > 64 &&
           (long long)g.B * g.H * g.W * g.C < (1ll << 31) &&
           (long long)g.L * (g.F / 128) * ((g.B + 127) / 128) * 16 < (1ll << 31);
}

// workspace that lets lc_forward cut the contraction of a layer with few fields into slices (0: not needed)
size_t forward_wide_workspace_bytes(const Geom &g) {
    if (!forward_wide_supported(g)) return 0;
    const int ns = wide_slices(g);
    return ns > 1 ? (size_t)ns * g.B * g.L * g.F * sizeof(float) : 0;
}

int launch_forward_wide_f32(const Geom &g, const float *x, const float *w, const float *bias, float alpha,
                            const float *alpha_dev, float *y, void *ws, size_t ws_bytes, hipStream_t s) {
    if (!forward_wide_supported(g)) return LC_EUNSUPPORTED;
    // 128-image tiles measured faster than 256-image ones here (1062 vs 1116 us on 256 x 64x64x32, 128 filters)
    int ns = wide_slices(g);
    if (ns > 1 && (!ws || ws_bytes < forward_wide_workspace_bytes(g))) ns = 1;   // no workspace: one slice
    // batch tile of 128, 96 or 64 images: the one that pads the batch least, the larger one on a tie (B = 192: two
    // tiles of 128 waste a quarter of the MFMAs); 16-value chunks stage two rows per thread, which rules 96 out
    const bool k32 = chunk_floats(g) == 32;
    const int mt = batch_tile_mt(g.B, k32);
    if (k32) {
        if (mt == 2) return launch_wide<32, 2>(g, x, w, bias, alpha, alpha_dev, y, (float *)ws, ns, s);
        if (mt == 3) return launch_wide<32, 3>(g, x, w, bias, alpha, alpha_dev, y, (float *)ws, ns, s);
        return launch_wide<32>(g, x, w, bias, alpha, alpha_dev, y, (float *)ws, ns, s);
    }
    if (mt == 2) return launch_wide<16, 2>(g, x, w, bias, alpha, alpha_dev, y, (float *)ws, ns, s);
    return launch_wide<16>(g, x, w, bias, alpha, alpha_dev, y, (float *)ws, ns, s);
}

}  // namespace lc
