// bf16 operands on the layers whose patch rows are not multiples of 16 values or whose filters come in blocks of 16
// or 32: lc_forward with the strip-sharing decomposition of the fp32 pipelined kernel
// (Sec. 3.1's untied fields overlap by R-S pixels, so a strip of adjacent fields shares the image rows it reads) and
// v_mfma_f32_16x16x16_bf16 in place of the fp32 matrix instruction.
//
// Workgroup = NLOC adjacent fields of one field row x a batch tile of 16*MT images x NW/NLOC blocks of 16*NT filters.
// A chunk is CQ values of one patch row for all fields of the strip, staged in LDS as bf16 (8-byte stores and reads);
// the next chunk's strip travels through registers meanwhile.  The contraction runs in blocks of 16 patch values:
// lane (m,kk) reads the four values 16 blk + 4 kk .. +3 of image m from LDS; lane (n,kk) loads the NT filters
// f0 + NT n .. of the four weight rows 16 blk + 4 kk .. +3 (the filters are the fast index of w, the patch values the
// slow one) and transposes them in registers into NT operands of four consecutive patch values each.  A patch row
// that is not a multiple of 16 ends in a partial block: its lanes beyond the row feed zeros as weights (the LDS
// holds the neighbouring field's pixels there).  The weights of a whole chunk are in flight ahead of their use.
#include <algorithm>

#include "lc_common.hpp"

namespace lc {
namespace {

constexpr int kStripSlots = 12;   // 8-byte staging registers per lane: chunk <= 12 * 256 * 8 B = 24 KB

// o[u] = (r[0].e_u, r[1].e_u, r[2].e_u, r[3].e_u): four rows of NT bf16 each -> NT operands of four rows
template <int NT>
__device__ __forceinline__ void rows_to_operands(const typename RawVec<bf16_t, NT>::V (&r)[4], u32x2 (&o)[NT]) {
    constexpr unsigned LO = 0x05040100u, HI = 0x07060302u;   // low / high halves of {src0:src1}
    if constexpr (NT == 1) {
        o[0] = (u32x2){(unsigned)r[0] | ((unsigned)r[1] << 16), (unsigned)r[2] | ((unsigned)r[3] << 16)};
    } else if constexpr (NT == 2) {
        o[0] = (u32x2){__builtin_amdgcn_perm(r[1], r[0], LO), __builtin_amdgcn_perm(r[3], r[2], LO)};
        o[1] = (u32x2){__builtin_amdgcn_perm(r[1], r[0], HI), __builtin_amdgcn_perm(r[3], r[2], HI)};
    } else {
        o[0] = (u32x2){__builtin_amdgcn_perm(r[1][0], r[0][0], LO), __builtin_amdgcn_perm(r[3][0], r[2][0], LO)};
        o[1] = (u32x2){__builtin_amdgcn_perm(r[1][0], r[0][0], HI), __builtin_amdgcn_perm(r[3][0], r[2][0], HI)};
        o[2] = (u32x2){__builtin_amdgcn_perm(r[1][1], r[0][1], LO), __builtin_amdgcn_perm(r[3][1], r[2][1], LO)};
        o[3] = (u32x2){__builtin_amdgcn_perm(r[1][1], r[0][1], HI), __builtin_amdgcn_perm(r[3][1], r[2][1], HI)};
    }
}

template <int MT, int NT, int NLOC, int NB, int NW>
__global__ __launch_bounds__(64 * NW, NT == 4 ? 2 : 3) void lc_forward_bf16_strip_kernel(Geom g, const bf16_t *__restrict__ x,
                                                                            const bf16_t *__restrict__ w,
                                                                            const float *__restrict__ bias, float alpha,
                                                                            float *__restrict__ y, int strips_per_row,
                                                                            int CQ, int sq4, int RS, int nbt,
                                                                            int work_first) {
    typedef typename RawVec<bf16_t, NT>::V WV;    // NT consecutive filters of one weight row
    typedef typename FVec<NT>::T OV;              // NT consecutive outputs
    typedef const __attribute__((address_space(1))) WV *gw_ptr;
    typedef const __attribute__((address_space(1))) u32x2 *gx4_ptr;
    typedef const __attribute__((address_space(1))) bf16_t *gt_ptr;
    constexpr int BT = 16 * MT, NFW = NW / NLOC, NTHR = 64 * NW;
    extern __shared__ __attribute__((aligned(16))) bf16_t xh[];      // [BT][RS]: the staged strip of one chunk
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, kk = lane >> 4;
    // batch tiles of one strip are neighbours in dispatch order on the same XCD
    const int t_id = remap_xcd(blockIdx.x, gridDim.x);
    const int work = work_first + t_id / nbt;
    const int i = work / strips_per_row, j0 = (work - i * strips_per_row) * NLOC;
    const int b0 = (t_id % nbt) * BT;
    const int wl = wave % NLOC, wf = wave / NLOC;
    const int j = j0 + wl;
    const int f0 = (blockIdx.y * NFW + wf) * NT * 16;
    const bool active = j < g.LW;
    const int loc = i * g.LW + (active ? j : g.LW - 1);   // idle waves shadow the last field of the row
    const int SC = g.S * g.C, WC = g.W * g.C;
    const size_t img = (size_t)g.H * WC;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int u = 0; u < NT; ++u) acc[mt][u] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // staging map: slot q of this thread copies 4-value vector number e = tid + NTHR*q of the [BT][sq4] chunk.
    // sb[q] = image << 16 | value offset in the row; bit 31: past the end of the chunk, bit 30: image beyond B.
    const int sqc = sq4 * 4;
    const int nslots = (BT * sq4 + NTHR - 1) / NTHR;
    int sb[kStripSlots];
    {
        int vv = tid % sq4, b = tid / sq4;
        const int dv = NTHR % sq4, db = NTHR / sq4;
#pragma unroll
        for (int q = 0; q < kStripSlots; ++q) {
            sb[q] = (b << 16) | (vv * 4);
            if (b >= BT) sb[q] = (int)0x80000000;
            else if (b0 + b >= g.B) sb[q] |= 0x40000000;
            vv += dv; b += db;
            if (vv >= sq4) { vv -= sq4; ++b; }
        }
    }
    // a partial last block reads up to 12 values past the staged row: those lanes' weights are zeros, and the LDS
    // there is cleared once so that no stale bit pattern (a NaN) meets them
    for (int e = tid; e < BT * 4; e += NTHR) *(u32x2 *)(xh + (e >> 2) * RS + sqc + 4 * (e & 3)) = (u32x2){0u, 0u};
    const int col0 = j0 * SC;
    u32x2 st[kStripSlots];
    auto stage_load = [&](int kh, int sc) {
        const bf16_t *row = x + (size_t)b0 * img + (size_t)(i * g.S + kh) * WC + col0 + sc * CQ;
        const int lim = WC - col0 - sc * CQ;          // values of this image row that exist from the chunk start on
#pragma unroll
        for (int q = 0; q < kStripSlots; ++q) {
            if (q < nslots) {
                const int b = (sb[q] >> 16) & 0x3fff, v = sb[q] & 0xffff;
                u32x2 t = (u32x2){0u, 0u};
                if ((sb[q] & 0xc0000000) == 0 && v < lim) t = *(gx4_ptr)(row + (size_t)b * img + v);
                st[q] = t;
            }
        }
    };
    auto stage_store = [&]() {
#pragma unroll
        for (int q = 0; q < kStripSlots; ++q) {
            if (q < nslots && sb[q] >= 0) {
                const int b = (sb[q] >> 16) & 0x3fff, v = sb[q] & 0xffff;
                *(u32x2 *)(xh + b * RS + v) = st[q];
            }
        }
    };

    // weights of block blk of the chunk that starts at patch value kbase: rows kbase + 16 blk + 4 kk + jj, clamped
    // into the field's matrix (rows beyond the patch row are multiplied by zeros or zeroed below)
    gt_ptr wfield = (gt_ptr)w + (size_t)loc * g.K * g.F + f0 + NT * n;
    WV wr[NB][4];
    auto load_block = [&](int kbase, int blk) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            int k = kbase + 16 * blk + 4 * kk + jj;
            k = k < g.K ? k : g.K - 1;
            wr[blk][jj] = *(gw_ptr)(wfield + (size_t)k * g.F);
        }
    };

    const bf16_t *xwin = xh + (size_t)(lane & 15) * RS + wl * SC + 4 * kk;
    const int nsub = g.RC / CQ, nchunks = g.R * nsub;
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
        if (16 * blk < CQ) load_block(0, blk);
    stage_load(0, 0);
    for (int c = 0; c < nchunks; ++c) {
        __syncthreads();                    // all waves are done reading the previous chunk
        stage_store();
        __syncthreads();
        const int cn = c + 1 < nchunks ? c + 1 : c;
        {
            const int kh = cn / nsub, sc = cn - kh * nsub;
            if (c + 1 < nchunks) stage_load(kh, sc);
        }
        const int knext = (cn / nsub) * g.RC + (cn % nsub) * CQ;
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            if (16 * blk < CQ) {            // uniform
                u32x2 a[MT], bo[NT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) a[mt] = *(const u32x2 *)(xwin + mt * 16 * RS + 16 * blk);
                rows_to_operands<NT>(wr[blk], bo);
                if (16 * blk + 4 * kk >= CQ) {   // lanes past the end of the patch row chunk
#pragma unroll
                    for (int u = 0; u < NT; ++u) bo[u] = (u32x2){0u, 0u};
                }
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int u = 0; u < NT; ++u) acc[mt][u] = mfma16_bf16(a[mt], bo[u], acc[mt][u]);
                load_block(knext, blk);
                // MFMAs and global loads keep their order (LDS reads and address arithmetic may move across)
                __builtin_amdgcn_sched_barrier(0x2 | 0x4 | 0x80);
            }
        }
    }

    if (!active) return;
    OV bv;
    if constexpr (NT == 1) bv = 0.f; else bv = (OV)(0.f);
    if (bias) bv = *(const OV *)(bias + (size_t)loc * g.F + f0 + NT * n);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int b = b0 + mt * 16 + 4 * kk + r;
            if (b >= g.B) continue;
            OV o;
            if constexpr (NT == 1) {
                o = alpha * acc[mt][0][r] + bv;
            } else {
#pragma unroll
                for (int u = 0; u < NT; ++u) o[u] = alpha * acc[mt][u][r] + bv[u];
            }
            *(OV *)(y + ((size_t)b * g.L + loc) * g.F + f0 + NT * n) = o;
        }
}

// row stride in bf16 values: 16 bytes past a multiple of 128 bytes, so that the 16 image rows a wave reads at once
// start four banks apart; the row keeps 16 values of padding behind the staged strip
int strip_row_stride(int sqc) { return ((sqc + 8 + 63) / 64) * 64 + 8; }   // at least 16 values of padding

// Host check of a lc_forward_bf16_strip_kernel launch.  tparam = {MT, NT, NLOC, NB, NW}; arg = {CQ, sq4, RS (bf16
// values), batch tiles, first strip, strips in this launch, strips per field row}.
int check_forward_bf16_strip(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0], NT = p.tparam[1], NLOC = p.tparam[2], NB = p.tparam[3], NW = p.tparam[4];
    const int CQ = p.arg[0], sq4 = p.arg[1], RS = p.arg[2], nbt = p.arg[3], first = p.arg[4], count = p.arg[5];
    const int strips = p.arg[6];
    LC_PLAN_REQUIRE(p, NLOC > 0 && NW % NLOC == 0 && (NT == 1 || NT == 2 || NT == 4));
    const int BT = 16 * MT, NFW = NW / NLOC, NTHR = 64 * NW, SC = g.S * g.C, WC = g.W * g.C, sqc = 4 * sq4;
    LC_PLAN_REQUIRE(p, (int)p.block == NTHR);
    // 8-byte accesses of four bf16 values: patch rows, image rows and field offsets in whole vectors
    LC_PLAN_REQUIRE(p, g.RC % 4 == 0 && WC % 4 == 0 && SC % 4 == 0);
    LC_PLAN_REQUIRE(p, g.F % (NFW * NT * 16) == 0 && (int)p.grid[1] == g.F / (NFW * NT * 16) && p.grid[2] == 1);
    // chunks of CQ values in NB blocks of 16 (the last one may be partial)
    LC_PLAN_REQUIRE(p, CQ > 0 && CQ % 4 == 0 && g.RC % CQ == 0 && NB == ceil_div(CQ, 16));
    LC_PLAN_REQUIRE(p, sqc >= CQ + (NLOC - 1) * SC && sqc <= 0xffff && BT <= 0x3fff);
    LC_PLAN_REQUIRE(p, (long long)BT * sq4 <= (long long)kStripSlots * NTHR);
    // a partial last block reads up to 12 values past a field's window; 16 values behind the staged row are cleared
    LC_PLAN_REQUIRE(p, RS % 4 == 0 && RS >= sqc + 16);
    LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)BT * RS * sizeof(bf16_t));
    LC_PLAN_REQUIRE(p, strips == ceil_div(g.LW, NLOC) && nbt == ceil_div(g.B, BT));
    LC_PLAN_REQUIRE(p, first >= 0 && count >= 1 && first + count <= strips * g.LH);
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] == (long long)count * nbt);
    return LC_OK;
}

template <int MT, int NT, int NB>
int launch_strip(const Geom &g, const bf16_t *x, const bf16_t *w, const float *bias, float alpha, float *y, int CQ,
                 int work_first, int work_count, hipStream_t s) {
    constexpr int NLOC = 4, NW = 4, BT = 16 * MT;
    const int sqc = (CQ + (NLOC - 1) * g.S * g.C + 3) & ~3;
    const int RS = strip_row_stride(sqc);
    const size_t lds = (size_t)BT * RS * sizeof(bf16_t);
    auto kern = lc_forward_bf16_strip_kernel<MT, NT, NLOC, NB, NW>;
    const int strips = (g.LW + NLOC - 1) / NLOC, nbt = (g.B + BT - 1) / BT;
    const long long nwg = (long long)work_count * nbt;
    if (nwg > 0x7fffffffLL) return LC_EUNSUPPORTED;
    dim3 grid((unsigned)nwg, g.F / (NT * 16));
    const LaunchPlan plan = make_plan("lc_forward_bf16_strip", {MT, NT, NLOC, NB, NW},
                                      {CQ, sqc / 4, RS, nbt, work_first, work_count, strips}, grid, 64 * NW, lds);
    if (int rc = check_forward_bf16_strip(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_forward (bf16 strip) launch", kern, s, g, x, w, bias, alpha, y, strips, CQ, sqc / 4, RS, nbt,
              work_first);
    return LC_OK;
}

// the chunk: the largest divisor of a patch row (in whole 4-value vectors, at most 128 values) whose strip fits the
// staging registers and 48 KB of LDS; 0 if none does
int strip_chunk(const Geom &g, int BT) {
    const int SC = g.S * g.C;
    for (int nsub = 1; nsub <= g.RC / 4; ++nsub) {
        if (g.RC % nsub) continue;
        const int CQ = g.RC / nsub;
        if (CQ % 4 || CQ > 128) continue;
        const int sqc = (CQ + 3 * SC + 3) & ~3;
        if ((size_t)BT * (sqc / 4) > (size_t)kStripSlots * 256) continue;
        if ((size_t)BT * strip_row_stride(sqc) * sizeof(bf16_t) > 48 * 1024) continue;
        if (sqc > 0xffff) continue;
        return CQ;
    }
    return 0;
}

template <int MT, int NT>
int launch_strip_nb(const Geom &g, const bf16_t *x, const bf16_t *w, const float *bias, float alpha, float *y, int CQ,
                    int first, int count, hipStream_t s) {
    switch ((CQ + 15) / 16) {
        case 1: return launch_strip<MT, NT, 1>(g, x, w, bias, alpha, y, CQ, first, count, s);
        case 2: return launch_strip<MT, NT, 2>(g, x, w, bias, alpha, y, CQ, first, count, s);
        case 3: return launch_strip<MT, NT, 3>(g, x, w, bias, alpha, y, CQ, first, count, s);
        case 4: return launch_strip<MT, NT, 4>(g, x, w, bias, alpha, y, CQ, first, count, s);
        case 5: return launch_strip<MT, NT, 5>(g, x, w, bias, alpha, y, CQ, first, count, s);
        case 6: return launch_strip<MT, NT, 6>(g, x, w, bias, alpha, y, CQ, first, count, s);
        case 7: return launch_strip<MT, NT, 7>(g, x, w, bias, alpha, y, CQ, first, count, s);
        default: return launch_strip<MT, NT, 8>(g, x, w, bias, alpha, y, CQ, first, count, s);
    }
}

// Batch tiles of 64 images: three workgroups fit a compute unit and the second tile of a strip finds the weights in
// L2.  128-image tiles (two per compute unit, one round of 512 plus a remainder launch where the strips do not fill a second round)
// measured slower: 114 against 106 us.
template <int NT>
int launch_strip_mt(const Geom &g, const bf16_t *x, const bf16_t *w, const float *bias, float alpha, float *y, int CQ,
                    hipStream_t s) {
    const int ntask = ((g.LW + 3) / 4) * g.LH;
    if (g.B > 32) return launch_strip_nb<4, NT>(g, x, w, bias, alpha, y, CQ, 0, ntask, s);
    return launch_strip_nb<2, NT>(g, x, w, bias, alpha, y, CQ, 0, ntask, s);
}

// ------------------------------------------------------------------------------ backward weights
// dw[l,k,f] = beta dw + sum_b x[b, patch k of l] dy[b,l,f] with bf16 operands (the weight gradient of Eq. 1's terms).
// The decomposition of the fp32 kernel: a wave owns one location, G*64 patch elements and 16*NT filters, both
// operands come straight from global memory with lanes along the contiguous axis (4 patch elements of an image row,
// NT filters).  The contraction runs over the batch, 16 images per bf16 MFMA: lane (m,kk) loads its vectors for the
// four images 4 kk .. +3 of a step and transposes them in registers, so that operand t holds patch element
// kg + 4 m + t (operand u: filter f0 + NT m + u) of those four images.  Loads run PF steps ahead in a register ring.
template <int G, int NT, int PF>
__global__ __launch_bounds__(256, 4) void lc_bwd_weights_bf16_rows_kernel(Geom g, const bf16_t *__restrict__ x,
                                                                       const bf16_t *__restrict__ dy, float beta,
                                                                       float *__restrict__ out, int kblocks,
                                                                       int ntasks) {
    typedef typename RawVec<bf16_t, NT>::V BR;     // NT consecutive dy values as loaded
    typedef typename FVec<NT>::T BV;               // NT consecutive outputs
    // the patch vectors are only element-aligned in general (a field starts every S*C elements)
    typedef __attribute__((address_space(1), aligned(2))) u32x2 GAV;
    typedef __attribute__((address_space(1))) BR GBV;
    typedef const __attribute__((address_space(1))) bf16_t *gt_ptr;
    constexpr int KB = G * 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, kk = lane >> 4;
    const int task = remap_xcd(blockIdx.x, gridDim.x) * 4 + wave;
    if (task >= ntasks) return;
    const int loc = task / kblocks, k0 = (task - loc * kblocks) * KB;
    const int i = loc / g.LW, j = loc - i * g.LW;
    const int f0 = blockIdx.y * NT * 16;
    const size_t img = (size_t)g.H * g.W * g.C, dyimg = (size_t)g.L * g.F;

    // rows of the A tiles beyond K are loaded from a valid address (element 0 of the patch) and never stored
    gt_ptr xa[G];
#pragma unroll
    for (int gg = 0; gg < G; ++gg) {
        const int k = k0 + gg * 64 + 4 * m;
        const int kc = k < g.K ? k : 0;
        const int kh = kc / g.RC, rem = kc - kh * g.RC;
        xa[gg] = (gt_ptr)x + (size_t)(4 * kk) * img + ((i * g.S + kh) * g.W + j * g.S) * g.C + rem;
    }
    gt_ptr da = (gt_ptr)dy + (size_t)(4 * kk) * dyimg + (size_t)loc * g.F + f0 + NT * m;

    f32x4 acc[G][4][NT];
#pragma unroll
    for (int gg = 0; gg < G; ++gg)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int u = 0; u < NT; ++u) acc[gg][t][u] = (f32x4){0.f, 0.f, 0.f, 0.f};

    u32x2 a[PF][G][4];
    BR bv[PF][4];
    auto load_step = [&](int ss) {      // one step = 16 images: this lane's four, then on to the next step
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
#pragma unroll
            for (int gg = 0; gg < G; ++gg) a[ss][gg][jj] = *(const GAV *)(xa[gg] + (size_t)jj * img);
            bv[ss][jj] = *(const GBV *)(da + (size_t)jj * dyimg);
        }
#pragma unroll
        for (int gg = 0; gg < G; ++gg) xa[gg] += 16 * img;
        da += 16 * dyimg;
    };
    auto mul_step = [&](int ss) {
        u32x2 bo[NT];
        rows_to_operands<NT>(bv[ss], bo);
#pragma unroll
        for (int gg = 0; gg < G; ++gg) {
            u32x2 ao[4];
            rows_to_operands<4>(a[ss][gg], ao);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int u = 0; u < NT; ++u) acc[gg][t][u] = mfma16_bf16(ao[t], bo[u], acc[gg][t][u]);
        }
    };
    const int nsteps = g.B >> 4;             // B % (16*PF) == 0 on this path
#pragma unroll
    for (int ss = 0; ss < PF; ++ss) load_step(ss);
    for (int s0 = PF; s0 < nsteps; s0 += PF) {
#pragma unroll
        for (int ss = 0; ss < PF; ++ss) {
            mul_step(ss);
            load_step(ss);
            // the refill of slot ss stays right behind the MFMAs that consumed it
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int ss = 0; ss < PF; ++ss) mul_step(ss);

    float *ol = out + (size_t)loc * g.K * g.F + f0 + NT * m;
#pragma unroll
    for (int gg = 0; gg < G; ++gg)
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int k = k0 + gg * 64 + 4 * (4 * kk + r) + t;
                if (k >= g.K) continue;
                BV *o = (BV *)(ol + (size_t)k * g.F);
                BV v;
                if constexpr (NT == 1) {
                    v = acc[gg][t][0][r];
                } else {
#pragma unroll
                    for (int u = 0; u < NT; ++u) v[u] = acc[gg][t][u][r];
                }
                if (beta != 0.f) v += beta * *o;
                *o = v;
            }
}

// Host check of a lc_bwd_weights_bf16_rows_kernel launch.  tparam = {G, NT, PF}; arg = {blocks of 64*G patch elements
// per field, wave tasks}.
int check_backward_weights_bf16_rows(const Geom &g, const LaunchPlan &p) {
    const int G = p.tparam[0], NT = p.tparam[1], PF = p.tparam[2];
    const int kblocks = p.arg[0], ntasks = p.arg[1];
    LC_PLAN_REQUIRE(p, p.block == 256 && (NT == 1 || NT == 2 || NT == 4));
    LC_PLAN_REQUIRE(p, g.RC % 4 == 0 && g.F % (NT * 16) == 0 && (int)p.grid[1] == g.F / (NT * 16) && p.grid[2] == 1);
    LC_PLAN_REQUIRE(p, PF >= 1 && g.B % (16 * PF) == 0);
    LC_PLAN_REQUIRE(p, kblocks == ceil_div(g.K, 64 * G) && (long long)ntasks == (long long)g.L * kblocks);
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] * 4 >= ntasks && (long long)(p.grid[0] - 1) * 4 < ntasks);
    LC_PLAN_REQUIRE(p, (long long)g.H * g.W * g.C < (1LL << 31));
    return LC_OK;
}

template <int G, int NT, int PF>
int launch_rows(const Geom &g, const bf16_t *x, const bf16_t *dy, float beta, float *out, hipStream_t s) {
    constexpr int KB = G * 64;
    const int kblocks = (g.K + KB - 1) / KB;
    const long long ntasks = (long long)g.L * kblocks;
    if (ntasks > (1LL << 30)) return LC_EUNSUPPORTED;
    dim3 grid((unsigned)((ntasks + 3) / 4), g.F / (NT * 16));
    const LaunchPlan plan = make_plan("lc_bwd_weights_bf16_rows", {G, NT, PF}, {kblocks, (int)ntasks}, grid, 256, 0);
    if (int rc = check_backward_weights_bf16_rows(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_backward_weights (bf16 rows) launch", (lc_bwd_weights_bf16_rows_kernel<G, NT, PF>), s, g, x, dy,
              beta, out, kblocks, (int)ntasks);
    return LC_OK;
}

// one step in flight and four waves per SIMD measured as fast as two steps and three waves (104 x 104 x 12 input, 10 x 10 fields, 32 filters, batch 128: 150 vs 153 us)
template <int G, int NT>
int launch_rows_pf(const Geom &g, const bf16_t *x, const bf16_t *dy, float beta, float *out, hipStream_t s) {
    return launch_rows<G, NT, 1>(g, x, dy, beta, out, s);
}

// The weight gradient with the patches shared through LDS.  In the kernel above every wave fetches its own
// 1200 x 128 patch, and those 8-byte loads are what binds it (same layer: 152 us, 88 us with the patch loads compiled out).
// Here a workgroup takes four adjacent fields and stages, per patch row, the image-row strip they share (as the
// forward kernel does; 2.5x fewer patch bytes on that layer, fetched once); wave = field.  Per patch row a wave contracts
// over the whole batch: lane (m,kk) reads the patch values 64 blk + 4 m .. +3 of the four images 16 s + 4 kk .. +3
// from LDS and transposes them in registers into four operands; the dy operands of all steps sit in registers for
// the whole kernel (batches up to 128 images).  The 64 x 16 NT tile of a patch row is stored as soon as it is
// complete.  Rows of a block beyond the patch row read the neighbour's pixels: they only reach output rows that
// are not stored.  The patch rows are split over grid.z so that small layers still fill the chip.
template <int NT, int NBK>
__global__ __launch_bounds__(256, 3) void lc_bwd_weights_bf16_strip_kernel(Geom g, const bf16_t *__restrict__ x,
                                                                         const bf16_t *__restrict__ dy, float beta,
                                                                         float *__restrict__ out, int strips_per_row,
                                                                         int sq4, int RS, int rows_per_wg) {
    typedef typename RawVec<bf16_t, NT>::V BR;     // NT consecutive dy values as loaded
    typedef typename FVec<NT>::T BV;               // NT consecutive outputs
    typedef const __attribute__((address_space(1))) BR *gb_ptr;
    typedef const __attribute__((address_space(1))) u32x2 *gx4_ptr;
    constexpr int BT = 128, NSTEP = BT / 16, NLOC = 4, NTHR = 256;
    extern __shared__ __attribute__((aligned(16))) bf16_t xh[];      // [BT][RS] (+ 64 values of slack)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, kk = lane >> 4;
    const int work = remap_xcd(blockIdx.x, gridDim.x);
    const int i = work / strips_per_row, j0 = (work - i * strips_per_row) * NLOC;
    const int j = j0 + wave;
    const bool active = j < g.LW;
    const int loc = i * g.LW + (active ? j : g.LW - 1);   // idle waves shadow the last field of the row
    const int f0 = blockIdx.y * NT * 16;
    const int kh_lo = blockIdx.z * rows_per_wg, kh_hi = min(g.R, kh_lo + rows_per_wg);
    const int SC = g.S * g.C, WC = g.W * g.C;
    const size_t img = (size_t)g.H * WC, dyimg = (size_t)g.L * g.F;

    // dy operands of every step: images 16 s + 4 kk .. +3, filters f0 + NT m .. (zeros beyond the batch)
    u32x2 bo[NSTEP][NT];
#pragma unroll
    for (int st = 0; st < NSTEP; ++st) {
        BR r[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int b = 16 * st + 4 * kk + jj;
            r[jj] = BR{};
            if (b < g.B) r[jj] = *(gb_ptr)(dy + (size_t)b * dyimg + (size_t)loc * g.F + f0 + NT * m);
        }
        rows_to_operands<NT>(r, bo[st]);
    }

    // staging map as in the forward kernel: slot q copies 4-value vector number tid + 256 q of the [BT][sq4] chunk
    const int sqc = sq4 * 4;
    const int nslots = (BT * sq4 + NTHR - 1) / NTHR;
    int sb[kStripSlots];
    {
        int vv = tid % sq4, b = tid / sq4;
        const int dv = NTHR % sq4, db = NTHR / sq4;
#pragma unroll
        for (int q = 0; q < kStripSlots; ++q) {
            sb[q] = (b << 16) | (vv * 4);
            if (b >= BT) sb[q] = (int)0x80000000;
            else if (b >= g.B) sb[q] |= 0x40000000;
            vv += dv; b += db;
            if (vv >= sq4) { vv -= sq4; ++b; }
        }
    }
    const int col0 = j0 * SC;
    u32x2 st[kStripSlots];
    auto stage_load = [&](int kh) {
        const bf16_t *row = x + (size_t)(i * g.S + kh) * WC + col0;
        const int lim = WC - col0;
#pragma unroll
        for (int q = 0; q < kStripSlots; ++q) {
            if (q < nslots) {
                const int b = (sb[q] >> 16) & 0x3fff, v = sb[q] & 0xffff;
                u32x2 t = (u32x2){0u, 0u};
                if ((sb[q] & 0xc0000000) == 0 && v < lim) t = *(gx4_ptr)(row + (size_t)b * img + v);
                st[q] = t;
            }
        }
    };
    auto stage_store = [&]() {
#pragma unroll
        for (int q = 0; q < kStripSlots; ++q) {
            if (q < nslots && sb[q] >= 0) {
                const int b = (sb[q] >> 16) & 0x3fff, v = sb[q] & 0xffff;
                *(u32x2 *)(xh + b * RS + v) = st[q];
            }
        }
    };

    const bf16_t *xwin = xh + (size_t)(4 * kk) * RS + wave * SC + 4 * m;
    float *ol = out + (size_t)loc * g.K * g.F + f0 + NT * m;
    const int nsteps = (g.B + 15) >> 4;
    if (kh_lo < kh_hi) stage_load(kh_lo);
    for (int kh = kh_lo; kh < kh_hi; ++kh) {
        __syncthreads();                    // all waves are done reading the previous patch row
        stage_store();
        __syncthreads();
        if (kh + 1 < kh_hi) stage_load(kh + 1);
#pragma unroll
        for (int blk = 0; blk < NBK; ++blk) {
            if (64 * blk >= g.RC) break;    // uniform
            f32x4 acc[4][NT];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int u = 0; u < NT; ++u) acc[t][u] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sp = 0; sp < NSTEP; ++sp) {
                if (sp < nsteps) {          // uniform
                    u32x2 r[4], ao[4];
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) r[jj] = *(const u32x2 *)(xwin + (size_t)(16 * sp + jj) * RS + 64 * blk);
                    rows_to_operands<4>(r, ao);
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int u = 0; u < NT; ++u) acc[t][u] = mfma16_bf16(ao[t], bo[sp][u], acc[t][u]);
                }
            }
            if (active) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const int kl = 64 * blk + 4 * (4 * kk + r) + t;
                        if (kl >= g.RC) continue;
                        BV *o = (BV *)(ol + (size_t)(kh * g.RC + kl) * g.F);
                        BV v;
                        if constexpr (NT == 1) {
                            v = acc[t][0][r];
                        } else {
#pragma unroll
                            for (int u = 0; u < NT; ++u) v[u] = acc[t][u][r];
                        }
                        if (beta != 0.f) v += beta * *o;
                        *o = v;
                    }
            }
        }
    }
}

// row stride: 16 bytes past a multiple of 128 bytes, wide enough for the staged strip and for the 64-value blocks of
// the last field (which read past its patch row)
int wstrip_row_stride(const Geom &g, int sqc) {
    const int nbk = (g.RC + 63) / 64, need = std::max(sqc, 3 * g.S * g.C + 64 * nbk);
    return ((need - 8 + 63) / 64) * 64 + 8;
}

// Host check of a lc_bwd_weights_bf16_strip_kernel launch.  tparam = {NT, NBK}; arg = {strips per field row, sq4, RS
// (bf16 values), patch rows per workgroup}.
int check_backward_weights_bf16_strip(const Geom &g, const LaunchPlan &p) {
    const int NT = p.tparam[0], NBK = p.tparam[1];
    const int strips = p.arg[0], sq4 = p.arg[1], RS = p.arg[2], rows_per_wg = p.arg[3];
    const int SC = g.S * g.C, WC = g.W * g.C, sqc = 4 * sq4;
    LC_PLAN_REQUIRE(p, p.block == 256 && (NT == 1 || NT == 2 || NT == 4));
    LC_PLAN_REQUIRE(p, g.RC % 4 == 0 && SC % 4 == 0 && WC % 4 == 0 && g.B <= 128);
    LC_PLAN_REQUIRE(p, g.F % (NT * 16) == 0 && (int)p.grid[1] == g.F / (NT * 16));
    // a patch row in NBK blocks of 64 values; the last field's blocks read past its patch row inside the LDS row
    LC_PLAN_REQUIRE(p, NBK * 64 >= g.RC);
    LC_PLAN_REQUIRE(p, sqc >= g.RC + 3 * SC && sqc <= 0xffff);
    LC_PLAN_REQUIRE(p, (long long)128 * sq4 <= (long long)kStripSlots * 256);
    LC_PLAN_REQUIRE(p, RS % 4 == 0 && RS >= sqc && RS >= 3 * SC + 64 * ceil_div(g.RC, 64));
    LC_PLAN_REQUIRE(p, p.lds_bytes >= ((size_t)128 * RS + 64) * sizeof(bf16_t));
    LC_PLAN_REQUIRE(p, strips == ceil_div(g.LW, 4) && (long long)p.grid[0] == (long long)strips * g.LH);
    LC_PLAN_REQUIRE(p, rows_per_wg >= 1 && (long long)p.grid[2] * rows_per_wg >= g.R &&
                           (long long)(p.grid[2] - 1) * rows_per_wg < g.R);
    return LC_OK;
}

template <int NT, int NBK>
int launch_wstrip(const Geom &g, const bf16_t *x, const bf16_t *dy, float beta, float *out, hipStream_t s) {
    const int sqc = (g.RC + 3 * g.S * g.C + 3) & ~3;
    const int RS = wstrip_row_stride(g, sqc);
    const size_t lds = ((size_t)128 * RS + 64) * sizeof(bf16_t);
    auto kern = lc_bwd_weights_bf16_strip_kernel<NT, NBK>;
    const int strips = (g.LW + 3) / 4;
    const long long nwork = (long long)strips * g.LH;
    if (nwork > 0x7fffffffLL) return LC_EUNSUPPORTED;
    // split the patch rows over grid.z until there are about four workgroups per compute unit
    int zsplit = 1;
    while (zsplit < g.R && nwork * (g.F / (NT * 16)) * zsplit < 4 * 256) ++zsplit;
    const int rows_per_wg = (g.R + zsplit - 1) / zsplit;
    dim3 grid((unsigned)nwork, g.F / (NT * 16), (g.R + rows_per_wg - 1) / rows_per_wg);
    const LaunchPlan plan = make_plan("lc_bwd_weights_bf16_strip", {NT, NBK}, {strips, sqc / 4, RS, rows_per_wg}, grid, 256, lds);
    if (int rc = check_backward_weights_bf16_strip(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_backward_weights (bf16 strip) launch", kern, s, g, x, dy, beta, out, strips, sqc / 4, RS,
              rows_per_wg);
    return LC_OK;
}

bool wstrip_supported(const Geom &g) {
    const int SC = g.S * g.C;
    if (g.RC % 4 || SC % 4 || (g.W * g.C) % 4 || g.F % 16 || g.B > 128 || g.RC > 128) return false;
    const int sqc = (g.RC + 3 * SC + 3) & ~3;
    if ((size_t)128 * (sqc / 4) > (size_t)kStripSlots * 256) return false;
    return ((size_t)128 * wstrip_row_stride(g, sqc) + 64) * sizeof(bf16_t) <= 48 * 1024 && sqc <= 0xffff;
}

template <int NT>
int launch_wstrip_nbk(const Geom &g, const bf16_t *x, const bf16_t *dy, float beta, float *out, hipStream_t s) {
    if (g.RC <= 64) return launch_wstrip<NT, 1>(g, x, dy, beta, out, s);
    return launch_wstrip<NT, 2>(g, x, dy, beta, out, s);
}

}  // namespace

// Shapes: patch rows in whole 4-value vectors, filters in blocks of 16, and either batches in steps of 16 images or
// a shape the strip-sharing kernel takes (any batch up to 128: it stages the missing images as zeros).
bool bf16_rows_backward_weights_supported(const Geom &g) {
    return g.RC % 4 == 0 && g.F % 16 == 0 && (g.B % 16 == 0 || wstrip_supported(g));
}

int launch_backward_weights_bf16_rows(const Geom &g, const void *xv, const void *dyv, float beta, float *dw,
                                      hipStream_t s) {
    if (!bf16_rows_backward_weights_supported(g)) return LC_EUNSUPPORTED;
    const bf16_t *x = (const bf16_t *)xv, *dy = (const bf16_t *)dyv;
    if (wstrip_supported(g)) {
        if (g.F % 32 == 0) return launch_wstrip_nbk<2>(g, x, dy, beta, dw, s);
        return launch_wstrip_nbk<1>(g, x, dy, beta, dw, s);
    }
    if (g.F % 64 == 0) return launch_rows_pf<1, 4>(g, x, dy, beta, dw, s);
    if (g.F % 32 == 0) return launch_rows_pf<2, 2>(g, x, dy, beta, dw, s);
    return launch_rows_pf<2, 1>(g, x, dy, beta, dw, s);
}

// Shapes: patch rows, field offsets and image rows in whole 4-value vectors (8-byte accesses), filters in blocks of 16.
bool bf16_strip_forward_supported(const Geom &g) {
    const int SC = g.S * g.C;
    if (g.RC % 4 || SC % 4 || (g.W * g.C) % 4 || g.F % 16 || g.B <= 16) return false;
    return strip_chunk(g, g.B > 32 ? 64 : 32) != 0;
}

int launch_forward_bf16_strip(const Geom &g, const void *xv, const void *wv, const float *bias, float alpha, float *y,
                              hipStream_t s) {
    if (!bf16_strip_forward_supported(g)) return LC_EUNSUPPORTED;
    const bf16_t *x = (const bf16_t *)xv, *w = (const bf16_t *)wv;
    const int CQ = strip_chunk(g, g.B > 32 ? 64 : 32);
    if (g.F % 64 == 0) return launch_strip_mt<4>(g, x, w, bias, alpha, y, CQ, s);
    if (g.F % 32 == 0) return launch_strip_mt<2>(g, x, w, bias, alpha, y, CQ, s);
    return launch_strip_mt<1>(g, x, w, bias, alpha, y, CQ, s);
}

}  // namespace lc
