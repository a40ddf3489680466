// lc_backward_data for layers whose S x S x C cells hold a multiple of 128 values (Eq. 1's decoder term):
// the workgroup tiling of the wide forward kernel with the operands' roles changed.
//
// A workgroup owns one cell of the input (128 of its values) and a batch tile of 32*MT images; its four waves
// form a 2 x 2 grid (16*MT images x 64 cell values).  The contraction runs over the fields that cover the cell
// and over their filters.  A chunk is 32 filters of one field: 128 contiguous bytes of dy per image, staged
// through LDS (two buffers, one barrier per chunk).  The filters are contiguous in memory along the contraction
// index: lane (n, kk) loads filters 16h + 4kk .. +3 of the weight row that cell value n has in the field, and
// lane (m, kk) reads the same four filters of image m from LDS, component t of both being MFMA step t.  Fields
// outside the grid are not in the chunk list; a cell no field covers gets zeros.
#include "lc_common.hpp"

namespace lc {

namespace {

typedef const __attribute__((address_space(1))) f32x4 *g4_ptr;
typedef const __attribute__((address_space(1))) float *gf_ptr;

constexpr int kChunk = 32;          // filters per LDS chunk
constexpr int kRowFloats = 36;      // 32 floats of a chunk + 4: eight rows' 16-byte reads cover all banks

// DENSE: a layer of one field that covers its whole input (R = H = W, the dense last layer of Sec. 3.1).  Every
// input value then has the same single covering field, so a "cell" is any block of 128 consecutive values k and
// dx[b][k] = sum_f w[k][f] dy[b][f].
template <int MT, int PD, bool DENSE>
__global__ __launch_bounds__(256, 2) void lc_bwd_data_wide_kernel(Geom g, const float *__restrict__ dy,
                                                                  const float *__restrict__ w,
                                                                  float *__restrict__ dx, int CW, int nblk,
                                                                  int btiles) {
    static_assert(PD == 1 || PD == 2, "one or two chunks of lookahead");
    constexpr int BT = 32 * MT, NS = MT;
    constexpr int BUF = BT * kRowFloats;
    extern __shared__ __attribute__((aligned(16))) float xs[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, kk = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    int t_id = remap_xcd(blockIdx.x, gridDim.x);
    const int bt = t_id % btiles;
    t_id /= btiles;
    const int nb = DENSE ? 0 : t_id % nblk, cell = DENSE ? t_id : t_id / nblk;
    const int ri = DENSE ? 0 : cell / CW, wi = DENSE ? 0 : cell - ri * CW;
    const int b0 = bt * BT;
    const int SC = g.S * g.C, AP = g.R / g.S;
    // fields (ri - a, wi - ap) inside the grid
    const int a_lo = max(0, ri - (g.LH - 1)), a_hi = min(AP - 1, ri);
    const int p_lo = max(0, wi - (g.LW - 1)), p_hi = min(AP - 1, wi);
    const int cpf = g.F / kChunk;
    const int nchunks = (a_hi >= a_lo && p_hi >= p_lo) ? (a_hi - a_lo + 1) * (p_hi - p_lo + 1) * cpf : 0;

    f32x4 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[mt][u] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // a cursor walks the chunk list in order and stays on the last chunk once it gets there
    struct Cursor { int a, ap, hf; };
    auto advance = [&](Cursor &q) {
        if (q.a == a_hi && q.ap == p_hi && q.hf == cpf - 1) return;
        if (++q.hf == cpf) {
            q.hf = 0;
            if (++q.ap > p_hi) { q.ap = p_lo; ++q.a; }
        }
    };

    const int seg = tid & 7, brow = tid >> 3;
    const int LF = g.L * g.F;
    int doff[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) doff[s] = min(b0 + brow + 32 * s, g.B - 1) * LF + seg * 4;
    Cursor sq = {a_lo, p_lo, 0};
    auto stage_load = [&](f32x4 (&st)[NS]) {
        const int o = ((ri - sq.a) * g.LW + (wi - sq.ap)) * g.F + sq.hf * kChunk;
#pragma unroll
        for (int s = 0; s < NS; ++s) st[s] = *(g4_ptr)((gf_ptr)dy + doff[s] + o);
        advance(sq);
    };
    auto stage_store = [&](int buf, const f32x4 (&st)[NS]) {
#pragma unroll
        for (int s = 0; s < NS; ++s) *(f32x4 *)(xs + buf * BUF + (brow + 32 * s) * kRowFloats + seg * 4) = st[s];
    };
    // weight row of this lane's cell value in tile nt, relative to the cell's corner in a field
    int kn[4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        const int nn = nb * 128 + wn * 64 + nt * 16 + n;
        const int dr = nn / SC;
        kn[nt] = (dr * g.RC + (nn - dr * SC)) * g.F + 4 * kk;
        // dense: row k of the only K x F matrix (rows beyond K repeat the last one and are not stored)
        if (DENSE) kn[nt] = min(cell * 128 + wn * 64 + nt * 16 + n, g.K - 1) * g.F + 4 * kk;
    }
    Cursor wq = {a_lo, p_lo, 0};
    int wh = 0;
    auto wload = [&](f32x4 (&r)[4]) {
        const size_t loc = (size_t)((ri - wq.a) * g.LW + (wi - wq.ap));
        gf_ptr p = (gf_ptr)w + (loc * g.K + (size_t)g.S * wq.a * g.RC + g.S * wq.ap * g.C) * g.F + wq.hf * kChunk +
                   16 * wh;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) r[nt] = *(g4_ptr)(p + kn[nt]);
        if (wh == 1) advance(wq);
        wh ^= 1;
    };

    if (nchunks > 0) {
        f32x4 st[PD][NS];
        f32x4 wr[2 * PD][4];
#pragma unroll
        for (int q = 0; q < 2 * PD; ++q) wload(wr[q]);
        stage_load(st[0]);
        stage_store(0, st[0]);
#pragma unroll
        for (int p = 0; p < PD; ++p) stage_load(st[p]);          // set p: chunk p+1
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
                        for (int nt = 0; nt < 4; ++nt) bo[nt] = wr[2 * sp + h][nt];
                        wload(wr[2 * sp + h]);
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            const f32x4 a = *(const f32x4 *)(ab + mt * 16 * kRowFloats + 16 * h);
#pragma unroll
                            for (int t = 0; t < 4; ++t)
#pragma unroll
                                for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = mfma16(a[t], bo[nt][t], acc[mt][nt]);
                        }
                    }
                    if (c + 1 < nchunks) stage_store(p ^ 1, st[sp]);
                    if (c + 1 + PD < nchunks) stage_load(st[sp]);
                }
                __syncthreads();
            }
        }
    }

#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        const int nn = nb * 128 + wn * 64 + nt * 16 + n;
        const int dr = nn / SC, rem = nn - dr * SC;
        const int row = ri * g.S + dr, col = wi * g.S + rem / g.C;
        size_t pix = ((size_t)row * g.W + wi * g.S) * g.C + rem;
        if (DENSE) {
            const int k = cell * 128 + wn * 64 + nt * 16 + n;
            if (k >= g.K) continue;
            pix = (size_t)k;                     // R = H = W: the patch index is the pixel index
        } else if (row >= g.H || col >= g.W) {
            continue;
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int b = b0 + wm * 16 * MT + mt * 16 + 4 * kk + r;
                if (b < g.B) dx[(size_t)b * g.H * g.W * g.C + pix] = acc[mt][nt][r];
            }
    }
}

// Host check of a lc_bwd_data_wide_kernel launch.  tparam = {MT, PD, DENSE}; arg = {cells per row, 128-value blocks
// per cell, batch tiles}.
int check_backward_data_wide(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0], DENSE = p.tparam[2];
    const int CW = p.arg[0], nblk = p.arg[1], btiles = p.arg[2];
    const int BT = 32 * MT;
    LC_PLAN_REQUIRE(p, p.block == 256);
    LC_PLAN_REQUIRE(p, g.F % kChunk == 0 && btiles == ceil_div(g.B, BT));
    // 32-bit element offsets of dy and inside a field's K x F matrix
    LC_PLAN_REQUIRE(p, (long long)g.B * g.L * g.F < (1LL << 31) && (long long)g.K * g.F < (1LL << 31));
    long long cells;
    if (DENSE) {
        LC_PLAN_REQUIRE(p, g.L == 1 && g.R == g.H && g.R == g.W && nblk == 1);
        cells = ceil_div(g.K, 128);
    } else {
        LC_PLAN_REQUIRE(p, g.R % g.S == 0 && (g.S * g.S * g.C) % 128 == 0 && nblk == g.S * g.S * g.C / 128);
        LC_PLAN_REQUIRE(p, CW == ceil_div(g.W, g.S));
        cells = (long long)ceil_div(g.H, g.S) * CW;
    }
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] == cells * nblk * btiles && p.grid[1] == 1 && p.grid[2] == 1);
    LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)2 * BT * kRowFloats * sizeof(float));
    return LC_OK;
}

template <int MT, int PD, bool DENSE>
int launch_wide(const Geom &g, const float *dy, const float *w, float *dx, hipStream_t s) {
    constexpr int BT = 32 * MT;
    const size_t lds = (size_t)2 * BT * kRowFloats * sizeof(float);
    auto kern = lc_bwd_data_wide_kernel<MT, PD, DENSE>;
    const int CH = (g.H + g.S - 1) / g.S, CW = (g.W + g.S - 1) / g.S;
    const int nblk = DENSE ? 1 : g.S * g.S * g.C / 128, btiles = (g.B + BT - 1) / BT;
    const long long cells = DENSE ? (g.K + 127) / 128 : (long long)CH * CW;
    const LaunchPlan plan = make_plan("lc_bwd_data_wide", {MT, PD, DENSE ? 1 : 0}, {CW, nblk, btiles},
                                      dim3((unsigned)(cells * nblk * btiles)), 256, lds);
    if (int rc = check_backward_data_wide(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_backward_data (wide) launch", kern, s, g, dy, w, dx, CW, nblk, btiles);
    return LC_OK;
}

}  // namespace

bool backward_data_wide_supported(const Geom &g) {
    const long long cells = (long long)((g.H + g.S - 1) / g.S) * ((g.W + g.S - 1) / g.S);
    return g.R % g.S == 0 && g.F % kChunk == 0 && (g.S * g.S * g.C) % 128 == 0 && g.B > 64 &&
           (long long)g.B * g.L * g.F < (1ll << 31) && (long long)g.K * g.F < (1ll << 31) &&
           cells * (g.S * g.S * g.C / 128) * ((g.B + 127) / 128) < (1ll << 31);
}

// one field covering the whole input: any K, filters in chunks of 32
bool backward_data_dense_supported(const Geom &g) {
    return g.L == 1 && g.R == g.H && g.R == g.W && g.F % kChunk == 0 && g.B > 64 &&
           (long long)g.B * g.F < (1ll << 31) && (long long)g.K * g.F < (1ll << 31);
}

int launch_backward_data_wide_f32(const Geom &g, const float *dy, const float *w, float *dx, hipStream_t s) {
    // batch tile of 128, 96 or 64 images: the one that pads the batch least, the larger one on a tie (B = 192: two
    // tiles of 128 waste a quarter of the MFMAs)
    int mt = batch_tile_mt(g.B, true);
    const bool dense = backward_data_dense_supported(g);
    if (!dense && !backward_data_wide_supported(g)) return LC_EUNSUPPORTED;
    // a layer that gives fewer workgroups than the chip has compute units takes 64-image tiles where they pad the
    // batch no more: twice the workgroups, each half as long (a 23 x 23 x 32 input under 6 x 6 fields at stride 2,
    // 144 cells, batch 128: 27.6 -> 26.4 us; 32-image tiles: 29.0 us, the chunk pipeline's latency is what is left)
    {
        const long long cells = dense ? (g.K + 127) / 128
                                      : (long long)((g.H + g.S - 1) / g.S) * ((g.W + g.S - 1) / g.S) * (g.S * g.S * g.C / 128);
        const int bt = 32 * mt;
        if (mt > 2 && cells * ((g.B + bt - 1) / bt) < 256 && (g.B + 63) / 64 * 64 <= (g.B + bt - 1) / bt * bt) mt = 2;
    }
    if (mt == 2) return dense ? launch_wide<2, 2, true>(g, dy, w, dx, s) : launch_wide<2, 2, false>(g, dy, w, dx, s);
    if (mt == 3) return dense ? launch_wide<3, 2, true>(g, dy, w, dx, s) : launch_wide<3, 2, false>(g, dy, w, dx, s);
    return dense ? launch_wide<4, 2, true>(g, dy, w, dx, s) : launch_wide<4, 2, false>(g, dy, w, dx, s);
}

}  // namespace lc
