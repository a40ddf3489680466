// bf16-operand forward contraction, workgroup-tiled (Eq. 1 encoder term, Sec. 3.1 geometry).
//
// A workgroup owns one field, 128 of its filters and a batch tile of 16*MT*WM images; its waves form a
// WM x 2 grid (16*MT images x 64 filters each).  The field's patch rows reach the waves through LDS in
// chunks of 64 contraction indices (128 contiguous bytes per image, two buffers, one barrier per chunk);
// the filters go straight from global memory to registers, one step of 32 indices ahead: lane (n, kk)
// loads rows 8kk..8kk+7 of the step at filters 4n..4n+3 (16 lanes cover whole 128-byte lines) and two
// 4x4 register transposes turn them into the k-contiguous operands of v_mfma_f32_16x16x32_bf16 for the
// four filter tiles, in which column n of tile u is filter 4n+u.
#include <algorithm>

#include "lc_common.hpp"

namespace lc {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x2 *g2_ptr;
typedef const __attribute__((address_space(1))) u32x4 *g4_ptr;
typedef const __attribute__((address_space(1))) unsigned short *gh_ptr;

__device__ __forceinline__ f32x4 mfma32_bf16(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                   0, 0, 0);
}

// r[t] = four bf16 (columns e0..e3) of row t, t = 0..7.  o[u] = column e_u of the eight rows, row 0 lowest.
__device__ __forceinline__ void transpose8x4_bf16(const u32x2 (&r)[8], u32x4 (&o)[4]) {
    constexpr unsigned LO = 0x05040100u, HI = 0x07060302u;   // low / high halves of {src0:src1}
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        o[0][p] = __builtin_amdgcn_perm(r[2 * p + 1][0], r[2 * p][0], LO);
        o[1][p] = __builtin_amdgcn_perm(r[2 * p + 1][0], r[2 * p][0], HI);
        o[2][p] = __builtin_amdgcn_perm(r[2 * p + 1][1], r[2 * p][1], LO);
        o[3][p] = __builtin_amdgcn_perm(r[2 * p + 1][1], r[2 * p][1], HI);
    }
}

constexpr int kChunk = 64;          // contraction indices per LDS chunk
constexpr int kRowBytes = 144;      // 128 bytes of a chunk + 16: eight rows' 16-byte reads cover all banks

// PD = chunks of lookahead: PD register sets hold the patch chunks c+1 .. c+PD on their way to LDS and the
// filter ring holds the 2*PD steps after the current one, so a load has PD chunks of MFMA work to land.
template <int MT, int PD, int WM>
__global__ __launch_bounds__(128 * WM, 2) void lc_forward_bf16_tiled_kernel(Geom g, const unsigned short *__restrict__ x,
                                                                    const unsigned short *__restrict__ w,
                                                                    const float *__restrict__ bias, float alpha,
                                                                    float *__restrict__ y, int fblocks, int btiles) {
    static_assert(PD == 1 || PD % 2 == 0, "the chunk loop is unrolled PD times and alternates two LDS buffers");
    constexpr int BT = 16 * MT * WM, NS = MT;     // NS: 16-byte staging slots per thread and chunk
    constexpr int SR = 16 * WM;                   // image rows one staging slot of the workgroup covers
    constexpr int BUF = BT * kRowBytes;
    constexpr int UN = PD == 1 ? 2 : PD;          // chunks per trip of the unrolled loop
    extern __shared__ __attribute__((aligned(16))) unsigned char xs[];
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
    const int cpr = g.RC / kChunk, nchunks = g.R * cpr, nsteps = 2 * nchunks;

    f32x4 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[mt][u] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // staging: slot s moves 16 bytes (segment tid&7) of image (tid>>3) + SR s; images beyond the batch
    // repeat image B-1 and their results are never stored
    const int seg = tid & 7, brow = tid >> 3;
    int xoff[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int b = min(b0 + brow + SR * s, g.B - 1);
        xoff[s] = (b * g.H + i * g.S) * WC + j * g.S * g.C + seg * 8;
    }
    auto stage_load = [&](int c, u32x4 (&st)[NS]) {
        const int kh = c / cpr;
        const int o = kh * WC + (c - kh * cpr) * kChunk;
#pragma unroll
        for (int s = 0; s < NS; ++s) st[s] = *(g4_ptr)((gh_ptr)x + xoff[s] + o);
    };
    auto stage_store = [&](int buf, const u32x4 (&st)[NS]) {
#pragma unroll
        for (int s = 0; s < NS; ++s) *(u32x4 *)(xs + buf * BUF + (brow + SR * s) * kRowBytes + seg * 16) = st[s];
    };
    // filters: the chunks tile k contiguously, so step q covers rows 32q .. 32q+31 of the field's K x F matrix
    gh_ptr wl = (gh_ptr)w + (size_t)loc * g.K * g.F + f0 + 4 * n + (size_t)(8 * kk) * g.F;
    auto wload = [&](int q, u32x2 (&r)[8]) {
        gh_ptr p = wl + (size_t)(32 * min(q, nsteps - 1)) * g.F;
#pragma unroll
        for (int t = 0; t < 8; ++t) r[t] = *(g2_ptr)(p + t * g.F);
    };

    u32x4 st[PD][NS];
    u32x2 wr[2 * PD][8];
#pragma unroll
    for (int q = 0; q < 2 * PD; ++q) wload(q, wr[q]);
    stage_load(0, st[0]);
    stage_store(0, st[0]);
#pragma unroll
    for (int p = 0; p < PD; ++p) stage_load(min(p + 1, nchunks - 1), st[p]);      // set p: chunk p+1
    __syncthreads();
    const int arow = (wm * 16 * MT + n) * kRowBytes + 16 * kk;
    for (int c0 = 0; c0 < nchunks; c0 += UN) {
#pragma unroll
        for (int p = 0; p < UN; ++p) {
            const int c = c0 + p;               // chunk c lives in buffer p & 1 (c0 is even)
            const int sp = p % PD;              // register set that holds chunk c+1
            if (c < nchunks) {
                const unsigned char *ab = xs + (p & 1) * BUF + arow;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    u32x4 bo[4];
                    transpose8x4_bf16(wr[2 * sp + h], bo);
                    wload(2 * c + h + 2 * PD, wr[2 * sp + h]);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const u32x4 a = *(const u32x4 *)(ab + mt * 16 * kRowBytes + 64 * h);
#pragma unroll
                        for (int u = 0; u < 4; ++u) acc[mt][u] = mfma32_bf16(a, bo[u], acc[mt][u]);
                    }
                }
                // the other buffer was last read in chunk c-1, which every wave left at the previous barrier
                if (c + 1 < nchunks) stage_store((p + 1) & 1, st[sp]);
                if (c + 1 + PD < nchunks) stage_load(c + 1 + PD, st[sp]);
            }
            __syncthreads();
        }
    }

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

// Host check of a lc_forward_bf16_tiled_kernel launch.  tparam = {MT, PD, WM}; arg = {filter blocks, batch tiles}.
int check_forward_bf16_tiled(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0], WM = p.tparam[2];
    const int fblocks = p.arg[0], btiles = p.arg[1];
    const int BT = 16 * MT * WM;
    LC_PLAN_REQUIRE(p, (int)p.block == 128 * WM);
    // 128 filters per workgroup; patch rows in whole chunks of 64 values whose starts are 16-byte aligned
    LC_PLAN_REQUIRE(p, g.F % 128 == 0 && fblocks == g.F / 128 && g.RC % kChunk == 0);
    LC_PLAN_REQUIRE(p, (g.S * g.C) % 8 == 0 && (g.W * g.C) % 8 == 0);
    // the staging map: tid >> 3 covers 16*WM image rows per slot, MT slots
    LC_PLAN_REQUIRE(p, btiles == ceil_div(g.B, BT));
    LC_PLAN_REQUIRE(p, (long long)g.B * g.H * g.W * g.C < (1LL << 31));
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] == (long long)g.L * fblocks * btiles && p.grid[1] == 1 && p.grid[2] == 1);
    LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)2 * BT * kRowBytes);
    return LC_OK;
}

template <int MT, int PD, int WM>
int launch_tiled(const Geom &g, const void *x, const void *w, const float *bias, float alpha, float *y,
                 hipStream_t s) {
    constexpr int BT = 16 * MT * WM;
    const size_t lds = (size_t)2 * BT * kRowBytes;
    auto kern = lc_forward_bf16_tiled_kernel<MT, PD, WM>;
    const int fblocks = g.F / 128, btiles = (g.B + BT - 1) / BT;
    const LaunchPlan plan = make_plan("lc_forward_bf16_tiled", {MT, PD, WM}, {fblocks, btiles},
                                      dim3((unsigned)(g.L * fblocks * btiles)), 128 * WM, lds);
    if (int rc = check_forward_bf16_tiled(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_forward (bf16, tiled) launch", kern, s, g, (const unsigned short *)x, (const unsigned short *)w,
              bias, alpha, y, fblocks, btiles);
    return LC_OK;
}

// ------------------------------------------------------------------------------------------------------
// Backward data (Eq. 1 decoder term): the same tiling with the operands' roles changed.  A workgroup owns
// one S x S x C cell of the input (128 of its values) and a batch tile; the contraction runs over the
// fields that cover the cell and over their filters.  A chunk is 64 filters of one field: 128 contiguous
// bytes of dy per image, staged through LDS.  The filters are contiguous in memory along the contraction
// index, so lane (n, kk) loads the operand of cell value n as it is: 16 bytes at filters 32h + 8kk of
// the weight row that cell value has in the field.  Fields outside the grid are not in the chunk list; a
// cell no field covers gets zeros.
template <int MT, int PD>
__global__ __launch_bounds__(256, 2) void lc_bwd_data_bf16_tiled_kernel(Geom g, const unsigned short *__restrict__ dy,
                                                                     const unsigned short *__restrict__ w,
                                                                     float *__restrict__ dx, int CW, int nblk,
                                                                     int btiles) {
    static_assert(PD == 1 || PD % 2 == 0, "the chunk loop is unrolled PD times and alternates two LDS buffers");
    constexpr int BT = 32 * MT, NS = MT, SR = 32;
    constexpr int BUF = BT * kRowBytes;
    constexpr int UN = PD == 1 ? 2 : PD;
    extern __shared__ __attribute__((aligned(16))) unsigned char xs[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, kk = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    int t_id = remap_xcd(blockIdx.x, gridDim.x);
    const int bt = t_id % btiles;
    t_id /= btiles;
    const int nb = t_id % nblk, cell = t_id / nblk;
    const int ri = cell / CW, wi = cell - ri * CW;
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
    for (int s = 0; s < NS; ++s) doff[s] = min(b0 + brow + SR * s, g.B - 1) * LF + seg * 8;
    Cursor sq = {a_lo, p_lo, 0};
    auto stage_load = [&](u32x4 (&st)[NS]) {
        const int o = ((ri - sq.a) * g.LW + (wi - sq.ap)) * g.F + sq.hf * kChunk;
#pragma unroll
        for (int s = 0; s < NS; ++s) st[s] = *(g4_ptr)((gh_ptr)dy + doff[s] + o);
        advance(sq);
    };
    auto stage_store = [&](int buf, const u32x4 (&st)[NS]) {
#pragma unroll
        for (int s = 0; s < NS; ++s) *(u32x4 *)(xs + buf * BUF + (brow + SR * s) * kRowBytes + seg * 16) = st[s];
    };
    // weight row of this lane's cell value in tile nt, relative to the cell's corner in a field
    int kn[4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        const int nn = nb * 128 + wn * 64 + nt * 16 + n;
        const int dr = nn / SC;
        kn[nt] = (dr * g.RC + (nn - dr * SC)) * g.F + 8 * kk;
    }
    Cursor wq = {a_lo, p_lo, 0};
    int wh = 0;
    auto wload = [&](u32x4 (&r)[4]) {
        const size_t loc = (size_t)((ri - wq.a) * g.LW + (wi - wq.ap));
        gh_ptr p = (gh_ptr)w + (loc * g.K + (size_t)g.S * wq.a * g.RC + g.S * wq.ap * g.C) * g.F + wq.hf * kChunk +
                   32 * wh;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) r[nt] = *(g4_ptr)(p + kn[nt]);
        if (wh == 1) advance(wq);
        wh ^= 1;
    };

    if (nchunks > 0) {
        u32x4 st[PD][NS];
        u32x4 wr[2 * PD][4];
#pragma unroll
        for (int q = 0; q < 2 * PD; ++q) wload(wr[q]);
        stage_load(st[0]);
        stage_store(0, st[0]);
#pragma unroll
        for (int p = 0; p < PD; ++p) stage_load(st[p]);          // set p: chunk p+1
        __syncthreads();
        const int arow = (wm * 16 * MT + n) * kRowBytes + 16 * kk;
        for (int c0 = 0; c0 < nchunks; c0 += UN) {
#pragma unroll
            for (int p = 0; p < UN; ++p) {
                const int c = c0 + p;               // chunk c lives in buffer p & 1 (c0 is even)
                const int sp = p % PD;              // register set that holds chunk c+1
                if (c < nchunks) {
                    const unsigned char *ab = xs + (p & 1) * BUF + arow;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        u32x4 bo[4];
#pragma unroll
                        for (int nt = 0; nt < 4; ++nt) bo[nt] = wr[2 * sp + h][nt];
                        wload(wr[2 * sp + h]);
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            const u32x4 a = *(const u32x4 *)(ab + mt * 16 * kRowBytes + 64 * h);
#pragma unroll
                            for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = mfma32_bf16(a, bo[nt], acc[mt][nt]);
                        }
                    }
                    if (c + 1 < nchunks) stage_store((p + 1) & 1, st[sp]);
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
        if (row >= g.H || col >= g.W) continue;
        const size_t pix = ((size_t)row * g.W + wi * g.S) * g.C + rem;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int b = b0 + wm * 16 * MT + mt * 16 + 4 * kk + r;
                if (b < g.B) dx[(size_t)b * g.H * g.W * g.C + pix] = acc[mt][nt][r];
            }
    }
}

// Host check of a lc_bwd_data_bf16_tiled_kernel launch.  tparam = {MT, PD}; arg = {cells per row, 128-value blocks per
// cell, batch tiles}.
int check_backward_data_bf16_tiled(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0];
    const int CW = p.arg[0], nblk = p.arg[1], btiles = p.arg[2];
    const int BT = 32 * MT;
    LC_PLAN_REQUIRE(p, p.block == 256);
    LC_PLAN_REQUIRE(p, g.R % g.S == 0 && g.F % kChunk == 0 && (g.S * g.S * g.C) % 128 == 0);
    LC_PLAN_REQUIRE(p, nblk == g.S * g.S * g.C / 128 && CW == ceil_div(g.W, g.S) && btiles == ceil_div(g.B, BT));
    LC_PLAN_REQUIRE(p, (long long)g.B * g.L * g.F < (1LL << 31) && (long long)g.K * g.F < (1LL << 31));
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] == (long long)ceil_div(g.H, g.S) * CW * nblk * btiles && p.grid[1] == 1 &&
                           p.grid[2] == 1);
    LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)2 * BT * kRowBytes);
    return LC_OK;
}

template <int MT, int PD>
int launch_bwd_data_tiled(const Geom &g, const void *dy, const void *w, float *dx, hipStream_t s) {
    constexpr int BT = 32 * MT;
    const size_t lds = (size_t)2 * BT * kRowBytes;
    auto kern = lc_bwd_data_bf16_tiled_kernel<MT, PD>;
    const int CH = (g.H + g.S - 1) / g.S, CW = (g.W + g.S - 1) / g.S;
    const int nblk = g.S * g.S * g.C / 128, btiles = (g.B + BT - 1) / BT;
    const LaunchPlan plan = make_plan("lc_bwd_data_bf16_tiled", {MT, PD}, {CW, nblk, btiles},
                                      dim3((unsigned)(CH * CW * nblk * btiles)), 256, lds);
    if (int rc = check_backward_data_bf16_tiled(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_backward_data (bf16, tiled) launch", kern, s, g, (const unsigned short *)dy,
              (const unsigned short *)w, dx, CW, nblk, btiles);
    return LC_OK;
}

// ------------------------------------------------------------------------------------------------------
// Backward weights (gradient of Eq. 1 with respect to W): dW[k][f] = sum_b x[b][k] dy[b][f] per field.
// A workgroup owns one field, 128 filters and a range of 64-row blocks of k; its waves take the blocks in
// turn.  The batch is the contraction index and the slow index of both operands, so both need 8 x 4
// register transposes.  dy serves every row block: it is transposed once and kept in LDS as
// [filter][image], and the waves read their operands from there (filter f sits in row (f%4)*32 + f/4, so
// that a lane's four tiles are four consecutive filters and neither the staging writes nor the operand
// reads run into bank conflicts).  Patch values are private to a wave: lane (m, kk) loads images
// 8kk..8kk+7 of the step at k = 4m..4m+3, which makes row m of tile u the weight row 4m+u; the loads run
// RING steps ahead, across block boundaries.
template <int RING>
__global__ __launch_bounds__(256, 2) void lc_bwd_weights_bf16_tiled_kernel(Geom g, const unsigned short *__restrict__ x,
                                                                        const unsigned short *__restrict__ dy,
                                                                        float beta, float *__restrict__ out,
                                                                        int fblocks, int ksplit, int nst, int rowb) {
    extern __shared__ __attribute__((aligned(16))) unsigned char xs[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, kk = lane >> 4;
    int t_id = remap_xcd(blockIdx.x, gridDim.x);
    const int ks = t_id % ksplit;
    t_id /= ksplit;
    const int fb = t_id % fblocks, loc = t_id / fblocks;
    const int i = loc / g.LW, j = loc - i * g.LW;
    const int nkb = g.K / 64;
    const int kb_lo = (nkb * ks) / ksplit, kb_hi = (nkb * (ks + 1)) / ksplit;

    // dy of the field, transposed into LDS; images beyond the batch are zeros
    {
        const int fg = tid & 31;
        gh_ptr dl = (gh_ptr)dy + (size_t)loc * g.F + fb * 128 + 4 * fg;
        const size_t dyimg = (size_t)g.L * g.F;
        for (int bg = tid >> 5; bg < nst * 4; bg += 8) {
            u32x2 r[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int b = 8 * bg + t;
                r[t] = (u32x2){0u, 0u};
                if (b < g.B) r[t] = *(g2_ptr)(dl + (size_t)b * dyimg);
            }
            u32x4 o[4];
            transpose8x4_bf16(r, o);
#pragma unroll
            for (int c = 0; c < 4; ++c) *(u32x4 *)(xs + (c * 32 + fg) * rowb + bg * 16) = o[c];
        }
    }
    __syncthreads();

    // patch operand: a cursor (row block, step) that stays on the wave's last block once it gets there
    const int WC = g.W * g.C, img = g.H * WC;
    int ckb = min(kb_lo + wave, nkb - 1), csb = 0;
    auto xload = [&](u32x2 (&r)[8]) {
        const int k0 = ckb * 64, kh = k0 / g.RC;
        gh_ptr p = (gh_ptr)x + ((i * g.S + kh) * WC + j * g.S * g.C + (k0 - kh * g.RC) + 4 * n);
#pragma unroll
        for (int t = 0; t < 8; ++t) r[t] = *(g2_ptr)(p + (size_t)(min(32 * csb + 8 * kk + t, g.B - 1) * img));
        if (++csb == nst) {
            csb = 0;
            if (ckb + 4 < kb_hi) ckb += 4;
        }
    };
    u32x2 ring[RING][8];
#pragma unroll
    for (int p = 0; p < RING; ++p) xload(ring[p]);

    const unsigned char *bbase = xs + n * rowb + 16 * kk;
    for (int kb = kb_lo + wave; kb < kb_hi; kb += 4) {
        f32x4 acc[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < 8; ++v) acc[u][v] = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (int sb0 = 0; sb0 < nst; sb0 += RING) {
#pragma unroll
            for (int p = 0; p < RING; ++p) {
                u32x4 ao[4];
                transpose8x4_bf16(ring[p], ao);
                xload(ring[p]);
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const u32x4 bf = *(const u32x4 *)(bbase + ((v & 3) * 32 + (v >> 2) * 16) * rowb + (sb0 + p) * 64);
#pragma unroll
                    for (int u = 0; u < 4; ++u) acc[u][v] = mfma32_bf16(ao[u], bf, acc[u][v]);
                }
            }
        }
        float *ol = out + ((size_t)loc * g.K + (size_t)kb * 64) * g.F + fb * 128 + 4 * n;
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                f32x4 *o = (f32x4 *)(ol + (size_t)(4 * (4 * kk + r) + u) * g.F);
                f32x4 v0, v1;
#pragma unroll
                for (int c = 0; c < 4; ++c) { v0[c] = acc[u][c][r]; v1[c] = acc[u][4 + c][r]; }
                if (beta != 0.f) {
                    v0 += beta * o[0];
                    v1 += beta * o[16];
                    o[0] = v0;
                    o[16] = v1;
                } else {
                    stream_store(v0, &o[0]);
                    stream_store(v1, &o[16]);
                }
                // keeps the read-modify-write of one row from being hoisted over the others' (registers)
                __builtin_amdgcn_sched_barrier(0);
            }
    }
}

// Host check of a lc_bwd_weights_bf16_tiled_kernel launch.  tparam = {RING}; arg = {filter blocks, workgroups per
// (field, filter block), steps of 32 images, LDS row bytes}.
int check_backward_weights_bf16_tiled(const Geom &g, const LaunchPlan &p) {
    const int RING = p.tparam[0];
    const int fblocks = p.arg[0], ksplit = p.arg[1], nst = p.arg[2], rowb = p.arg[3];
    LC_PLAN_REQUIRE(p, p.block == 256);
    // 64-row blocks inside one patch row; 8-byte patch vectors; 128 filters per workgroup
    LC_PLAN_REQUIRE(p, g.RC % 64 == 0 && (g.S * g.C) % 4 == 0 && (g.W * g.C) % 4 == 0);
    LC_PLAN_REQUIRE(p, g.F % 128 == 0 && fblocks == g.F / 128);
    // the batch in whole ring turns of 32-image steps, all of it transposed into LDS
    LC_PLAN_REQUIRE(p, RING >= 1 && nst % RING == 0 && nst * 32 >= g.B && rowb >= nst * 64 && rowb % 16 == 0);
    LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)128 * rowb);
    // every wave of a workgroup has at least one row block
    LC_PLAN_REQUIRE(p, ksplit >= 1 && ksplit * 4 <= std::max(g.K / 64, 4));
    LC_PLAN_REQUIRE(p, (long long)g.B * g.H * g.W * g.C < (1LL << 31));
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] == (long long)g.L * fblocks * ksplit && p.grid[1] == 1 && p.grid[2] == 1);
    return LC_OK;
}

template <int RING>
int launch_bwd_weights_tiled(const Geom &g, const void *x, const void *dy, float beta, float *dw, hipStream_t s) {
    const int nst = ((g.B + 31) / 32 + RING - 1) / RING * RING;
    const int rowb = nst * 64 + 16;
    const size_t lds = (size_t)128 * rowb;
    auto kern = lc_bwd_weights_bf16_tiled_kernel<RING>;
    // split the row blocks of a field over 1..4 workgroups, whichever fills whole rounds of the chip best
    const int fblocks = g.F / 128, nkb = g.K / 64;
    const long long base = (long long)g.L * fblocks, slots = 512;
    int ksplit = 1;
    double best = 0.0;
    for (int ks = 1; ks <= 4 && ks * 4 <= nkb; ++ks) {
        const long long tasks = base * ks, rounds = (tasks + slots - 1) / slots;
        const double eff = (double)tasks / (double)(rounds * slots);
        if (eff > best + 0.02) { best = eff; ksplit = ks; }
    }
    const LaunchPlan plan = make_plan("lc_bwd_weights_bf16_tiled", {RING}, {fblocks, ksplit, nst, rowb},
                                      dim3((unsigned)(base * ksplit)), 256, lds);
    if (int rc = check_backward_weights_bf16_tiled(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_backward_weights (bf16, tiled) launch", kern, s, g, (const unsigned short *)x,
              (const unsigned short *)dy, beta, dw, fblocks, ksplit, nst, rowb);
    return LC_OK;
}

}  // namespace

// Shapes of the tiled kernel: filter blocks of 128, patch rows that split into 64-index chunks, 16-byte
// aligned chunk starts, and element offsets that fit 32 bits.
bool bf16_tiled_forward_supported(const Geom &g) {
    return g.F % 128 == 0 && g.RC % kChunk == 0 && (g.S * g.C) % 8 == 0 && (g.W * g.C) % 8 == 0 && g.B > 64 &&
           (long long)g.B * g.H * g.W * g.C < (1ll << 31) && (long long)g.L * g.F / 128 * ((g.B + 127) / 128) < (1ll << 31);
}

int launch_forward_bf16_tiled(const Geom &g, const void *x, const void *w, const float *bias, float alpha, float *y,
                              hipStream_t s) {
    if (!bf16_tiled_forward_supported(g)) return LC_EUNSUPPORTED;
    // 256-image tiles read the filters once; they fit two workgroups per CU only with one chunk of lookahead.
    // (Two adjacent fields in one 512-thread workgroup, sharing the staged chunks - five per patch row of the pair
    // instead of eight on a 64 x 64 x 32 input under 8 x 8 fields at stride 2 - asked L2 for a quarter less and still
    // measured 214 against 194 us: one workgroup per compute unit is one barrier domain with one chunk in flight,
    // where two independent workgroups cover each other's waits.)
    if (g.B > 128) return launch_tiled<8, 1, 2>(g, x, w, bias, alpha, y, s);
    return launch_tiled<4, 2, 2>(g, x, w, bias, alpha, y, s);
}

// Tiled backward data: fields that tile the cells exactly, filters in chunks of 64, cells of 128-value blocks.
bool bf16_tiled_backward_data_supported(const Geom &g) {
    const long long cells = (long long)((g.H + g.S - 1) / g.S) * ((g.W + g.S - 1) / g.S);
    return g.R % g.S == 0 && g.F % kChunk == 0 && (g.S * g.S * g.C) % 128 == 0 && g.B > 64 &&
           (long long)g.B * g.L * g.F < (1ll << 31) && (long long)g.K * g.F < (1ll << 31) &&
           cells * (g.S * g.S * g.C / 128) * ((g.B + 127) / 128) < (1ll << 31);
}

int launch_backward_data_bf16_tiled(const Geom &g, const void *dy, const void *w, float *dx, hipStream_t s) {
    if (!bf16_tiled_backward_data_supported(g)) return LC_EUNSUPPORTED;
    if (g.B > 128) return launch_bwd_data_tiled<8, 1>(g, dy, w, dx, s);
    return launch_bwd_data_tiled<4, 2>(g, dy, w, dx, s);
}

// Tiled backward weights: 64-row blocks inside one patch row, filter blocks of 128, a batch that fits LDS.
bool bf16_tiled_backward_weights_supported(const Geom &g) {
    return g.RC % 64 == 0 && g.F % 128 == 0 && (g.S * g.C) % 4 == 0 && (g.W * g.C) % 4 == 0 && g.B > 64 &&
           g.B <= 512 && (long long)g.B * g.H * g.W * g.C < (1ll << 31) && (long long)g.L * (g.F / 128) * 4 < (1ll << 31);
}

int launch_backward_weights_bf16_tiled(const Geom &g, const void *x, const void *dy, float beta, float *dw,
                                       hipStream_t s) {
    if (!bf16_tiled_backward_weights_supported(g)) return LC_EUNSUPPORTED;
    return launch_bwd_weights_tiled<2>(g, x, dy, beta, dw, s);
}

}  // namespace lc
