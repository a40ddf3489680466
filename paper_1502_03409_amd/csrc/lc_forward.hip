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

template <int MT, int NT, int NLOC, bool MASK, typename T>
__device__ __forceinline__ void fwd_row(f32x4 (&acc)[MT][NT], const float *__restrict__ xs_win, int rs,
                                        const T *__restrict__ wrow, int F, int RC, int kk, bool (&fok)[NT]) {
    const int lane_m = threadIdx.x & 15;
#pragma unroll 2
    for (int kq = 0; kq < RC; kq += 4) {
        float bw[NT], a[MT];
        const bool kok = !MASK || (kq + kk < RC);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (MASK)
                bw[nt] = (kok && fok[nt]) ? ld_f32(wrow + (size_t)kq * F + nt * 16) : 0.f;
            else
                bw[nt] = ld_f32(wrow + (size_t)kq * F + nt * 16);
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

// T: storage type of x and w (float, or bf16 bit patterns widened on their way in)
template <int MT, int NT, int NLOC, typename T>
__global__ __launch_bounds__(256) void lc_forward_kernel(Geom g, const T *__restrict__ x,
                                                         const T *__restrict__ w,
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
    const T *wl_base = w + (size_t)loc * g.K * g.F + f0 + n;
    const float *xs_win = xs + wl * g.S * g.C + kk;

    for (int kh = 0; kh < g.R; ++kh) {
        __syncthreads();
        {
            const T *xrow = x + (size_t)(i * g.S + kh) * g.W * g.C + col0;
            int q = q_first, bb = b_first;
            while (bb < BT) {
                float v = 0.f;
                if (q < nvalid && b0 + bb < g.B) v = ld_f32(xrow + (size_t)(b0 + bb) * img + q);
                xs[bb * rs + q] = v;
                q += dq;
                bb += db;
                if (q >= sq) { q -= sq; ++bb; }
            }
        }
        __syncthreads();
        if (active) {
            const T *wrow = wl_base + (size_t)(kh * g.RC + kk) * g.F;
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


// ---------------------------------------------------------------------------------------------
// Fast path (aligned shapes: patch rows, strides and filter counts that allow whole-line vector
// accesses).  Same decomposition as above, re-arranged so that the MFMA pipe never waits:
//   * the image strip of the NEXT chunk is fetched into registers (one dwordx4 per lane and slot)
//     while the current chunk is multiplied out of LDS; a chunk is CQ floats of one patch row for
//     all fields of the strip;
//   * the weights run ahead of their use in a register ring of UNR k-steps that is never drained:
//     w[l] is contiguous in k, so the ring simply walks through the whole K x F matrix of the field;
//   * lane (n,kk) of a weight load holds NT consecutive filters f0+NT*n.. of row k+kk, i.e. column n
//     of NT different N-tiles: 16 lanes cover a whole run of w, and the epilogue stores NT filters
//     of one image as one vector.
// Rows of A are images and are never masked (images beyond B are staged as zeros).
constexpr int kFwdStageSlotsWide = 6;   // eight-wave workgroups: half the registers per lane
constexpr int kFwdStageSlots = 12;  // dwordx4 staging registers per lane: chunk <= 12*256*16 B = 48 KB

template <int MT, int NT, int NLOC, int UNR, int NW = 4, typename T = float, int SPC = 0, int NRT = 1, int NSL = 0>
__global__ __launch_bounds__(64 * NW, NW == 8 ? 4 : 1) void lc_forward_fast_kernel(Geom g, const T *__restrict__ x,
                                                              const T *__restrict__ w,
                                                              const float *__restrict__ bias, float alpha,
                                                              const float *__restrict__ alpha_dev,
                                                              float *__restrict__ y, int strips_per_row, int CQ,
                                                              int sq4, int RS, int NR, int work_offset, int nbt) {
    typedef typename RawVec<T, NT>::V WV;     // NT consecutive weights as loaded
    typedef typename RawVec<T, 4>::V XV;      // four consecutive x values as loaded
    typedef typename FVec<NT>::T OV;          // NT consecutive outputs
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef const __attribute__((address_space(1))) WV *gw_ptr;
    typedef const __attribute__((address_space(1))) XV *gx4_ptr;
    typedef const __attribute__((address_space(1))) T *gt_ptr;
    constexpr int BT = 16 * MT, NFW = NW / NLOC, NTHR = 64 * NW;   // NW waves: NLOC fields x NFW filter blocks
    // staging slots per lane; NSL > 0 (with SPC > 0, where every slot loads): exactly as many as a chunk needs
    constexpr int SLOTS = NSL > 0 ? NSL : (NW == 8 ? kFwdStageSlotsWide : kFwdStageSlots);
    extern __shared__ __attribute__((aligned(16))) float xs[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, kk = lane >> 4;
    // batch tiles of one strip are neighbours in dispatch order on the same XCD: the later ones find
    // the strip's weights in that XCD's L2
    const int t_id = remap_xcd(blockIdx.x, gridDim.x);
    const int work = work_offset + t_id / nbt;
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

    // staging map: a chunk is NR patch rows x sq4 dwordx4 per image; slot q of this thread copies dwordx4
    // number e = tid + NTHR*q of the [BT][NR][sq4] chunk.  sb[q] = image << 16 | row << 12 | float offset in
    // the row; bit 31: past the end of the chunk (slot unused), bit 30: image beyond the batch (zeros).
    const int per_img = NR * sq4, sqc = sq4 * 4;
    const int nslots = (BT * per_img + NTHR - 1) / NTHR;
    int sb[SLOTS];
    {
        int vv = tid % per_img, b = tid / per_img;
        const int dv = NTHR % per_img, db = NTHR / per_img;
#pragma unroll
        for (int q = 0; q < SLOTS; ++q) {
            const int r = vv / sq4, v = vv - r * sq4;
            sb[q] = (b << 16) | (r << 12) | (v * 4);
            if (b >= BT) {
                // past the end of the chunk: unused, or (SPC > 0, every slot loads and stores) a second copy of the
                // chunk's last element
                sb[q] = SPC > 0 ? ((BT - 1) << 16) | ((NR - 1) << 12) | ((sq4 - 1) * 4) : (int)0x80000000;
            } else if (b0 + b >= g.B) {
                sb[q] |= 0x40000000;
            }
            vv += dv; b += db;
            if (vv >= per_img) { vv -= per_img; ++b; }
        }
    }
    const int col0 = j0 * SC;
    XV st[SLOTS];
    // SPC > 0 (k-steps per chunk known at compile time; one whole patch row per chunk, every staging slot in use):
    // every slot loads, from an address clamped into the image (what lands beyond the batch or the row only reaches
    // rows and waves that are not stored), and the k-step loop is unrolled, so the number of loads between a
    // chunk's staging loads and their use is a constant the compiler can wait on exactly.  With counts it cannot
    // see it waits for every outstanding load before the LDS stores and again before the chunk's first MFMA, which
    // drains the weight ring and exposes the staging loads' latency once per chunk.
    int so[SPC > 0 ? SLOTS : 1];
    if constexpr (SPC > 0) {
        const int lim0 = WC - col0;
#pragma unroll
        for (int q = 0; q < SLOTS; ++q) {
            const int b = (sb[q] >> 16) & 0x3fff, r = (sb[q] >> 12) & 15, v = sb[q] & 0xfff;
            so[q] = min(b, g.B - 1 - b0) * (int)img + r * WC + min(v, max(lim0 - 4, 0));
        }
    }
    auto stage_load = [&](int kh, int sc) {
        const T *row = x + (size_t)b0 * img + (size_t)(i * g.S + kh) * WC + col0 + sc * CQ;
        if constexpr (SPC > 0) {
#pragma unroll
            for (int q = 0; q < SLOTS; ++q) st[q] = *(gx4_ptr)(row + so[q]);
            return;
        }
        const int lim = WC - col0 - sc * CQ;          // floats of this image row that exist from the chunk start on
#pragma unroll
        for (int q = 0; q < SLOTS; ++q) {
            if (q < nslots) {
                const int b = (sb[q] >> 16) & 0x3fff, r = (sb[q] >> 12) & 15, v = sb[q] & 0xfff;
                XV t = XV{};
                if ((sb[q] & 0xc0000000) == 0 && v < lim) t = *(gx4_ptr)(row + (size_t)b * img + r * WC + v);
                st[q] = t;
            }
        }
    };
    auto stage_store = [&]() {
#pragma unroll
        for (int q = 0; q < SLOTS; ++q) {
            if (SPC > 0 || (q < nslots && sb[q] >= 0)) {   // SPC > 0: every slot is in use
                const int b = (sb[q] >> 16) & 0x3fff, r = (sb[q] >> 12) & 15, v = sb[q] & 0xfff;
                // rows of images 8..15 (mod 16) sit 2 floats to the right (see xwin below)
                float *dst = xs + b * RS + r * sqc + ((b >> 2) & 2) + v;
                const f32x4 f = raw_widen4<T>(st[q]);
                *(f32x2 *)dst = (f32x2){f[0], f[1]};
                *(f32x2 *)(dst + 2) = (f32x2){f[2], f[3]};
            }
        }
    };

    // weight ring: slot s holds k-step S = s (mod UNR); w[loc] is walked linearly in k
    const int nsteps = g.K >> 2;
    gw_ptr wp = (gw_ptr)(w + (size_t)loc * g.K * g.F + (size_t)kk * g.F + f0 + NT * n);
    const size_t wstep = (size_t)g.F;           // in units of float: 4 rows per k-step -> 4*F floats
    WV wr[UNR];
    int wleft = nsteps;                         // k-steps not yet requested
    if constexpr (SPC > 0) {
        stage_load(0, 0);
    }
#pragma unroll
    for (int s = 0; s < UNR; ++s) {
        wr[s] = *wp;
        --wleft;
        wp = (gw_ptr)((gt_ptr)wp + (wleft > 0 ? 4 * wstep : 0));
    }

    // LDS bank layout: RS == 4 (mod 32) puts images m and m+8 of an A operand on the same banks; shifting
    // the rows of images 8..15 by two floats makes the 32 (image, k) pairs of a half-wave hit 32 banks.
    const float *xwin = xs + (size_t)(lane & 15) * RS + ((lane >> 2) & 2) + wl * SC + kk;
    const int spc = CQ >> 2;                    // k-steps per patch row of a chunk, a multiple of UNR
    const int nsub = g.RC / CQ;                 // NR > 1 only with whole rows (nsub == 1)
    auto ksteps = [&](const float *xrow, int s0) {
#pragma unroll
        for (int ss = 0; ss < UNR; ++ss) {
            float a[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[mt] = xrow[mt * 16 * RS + 4 * (s0 + ss)];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int u = 0; u < NT; ++u)
                    acc[mt][u] = mfma16(a[mt], raw_get<T, NT>(wr[ss], u), acc[mt][u]);
            wr[ss] = *wp;
            --wleft;
            wp = (gw_ptr)((gt_ptr)wp + (wleft > 0 ? 4 * wstep : 0));
            // MFMAs and global loads keep their order (LDS reads and address arithmetic may move across)
            __builtin_amdgcn_sched_barrier(0x2 | 0x4 | 0x80);
        }
    };
    if constexpr (SPC > 0) {
        // One whole patch row per chunk.  The next chunk's staging loads go out after the first UNR k-steps: every
        // ring load that is still awaited then is younger than they are, so no wait on the ring has to cover them
        // (the counter retires loads in order), and they have the rest of the chunk to arrive.  They are always
        // issued (the last chunk loads its own row again): a path without them would make the compiler assume,
        // where the paths join, that none are in flight.  For the same reason a chunk's staging loads and the LDS
        // stores that use them sit in the same loop iteration: the compiler then sees every load between them.
        __syncthreads();
        stage_store();                          // chunk 0
        __syncthreads();
        for (int kh = 0; kh < g.R; kh += NRT) {          // NRT patch rows per chunk (R a multiple of NRT)
            ksteps(xwin, 0);
            stage_load(min(kh + NRT, g.R - NRT), 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s0 = UNR; s0 < SPC; s0 += UNR) ksteps(xwin, s0);
#pragma unroll
            for (int r = 1; r < NRT; ++r)
#pragma unroll
                for (int s0 = 0; s0 < SPC; s0 += UNR) ksteps(xwin + r * sqc, s0);
            __syncthreads();                    // all waves are done reading this chunk
            stage_store();                      // the next one (after the last chunk: its own row again, unused)
            __syncthreads();
        }
    } else {
        stage_load(0, 0);
        for (int kh = 0; kh < g.R; kh += NR) {
            for (int sc = 0; sc < nsub; ++sc) {
                __syncthreads();                    // all waves are done reading the previous chunk
                stage_store();
                __syncthreads();
                {
                    int nsc = sc + 1, nkh = kh;
                    if (nsc == nsub) { nsc = 0; nkh += NR; }
                    if (nkh < g.R) stage_load(nkh, nsc);
                }
                for (int r = 0; r < NR; ++r) {
                    const float *xrow = xwin + r * sqc;
                    for (int s0 = 0; s0 < spc; s0 += UNR) ksteps(xrow, s0);
                }
            }
        }
    }

    if (!active) return;
    if (alpha_dev) alpha = *alpha_dev;
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

// ---------------------------------------------------------------------------------------------
// The fast path for fp32 operands and whole patch rows per chunk, with a hand-kept memory schedule.  Same
// decomposition as lc_forward_fast_kernel (a workgroup is a strip of NLOC fields of one field row times a batch tile;
// a chunk is NRT patch rows of the strip; a k-step is one MFMA per accumulator); what differs:
//   - x goes from global memory straight into LDS (16 bytes per lane, lane i of a wave's load lands 16 i bytes past
//     the load's LDS base): no staging registers, no LDS stores.  A buffer is the batch tile's rows one after the
//     other, each NRT patch-row pieces of sq4 vectors (plus a pad vector where that makes the vector count odd: the
//     16 rows a wave reads at once then start four banks apart); vector P of the buffer belongs to lane P % NTHR of
//     load P / NTHR and comes from the same place in every chunk, relative to the chunk's first vector.  Every lane
//     loads: images past the batch and columns past the image row are clamped into x, where they only feed rows and
//     waves that store nothing; pad vectors and the slack behind the last row load the chunk's first vector.
//   - a lane's A operands of four k-steps are four consecutive floats of the patch row, one 16-byte LDS read where
//     the old order needed four 4-byte reads: k-step t of group gi contracts k = 16 gi + 4 kk + t instead of
//     16 gi + 4 t + kk (a sum over k: any order both operands agree on), so lane (n,kk) loads row
//     16 gi + 4 kk + t of w[l].  A patch row of SPC k-steps is SPC/4 such groups and a tail group of SPC%4 steps
//     (k = 16 (SPC/4) + (SPC%4) kk + t).
//   - weight pointers are scalar (the wave index is read into a scalar register; a lane adds its fixed offset), and
//     the loads are inline assembly with every wait written out.  The memory counter counts loads in program order:
//         chunk c:  [NSLOT x loads of chunk c+1]  then per k-step p: wait, MFMAs, [one weight load, of k-step p+U]
//     so the weights of k-step p are followed by U-1 younger weight loads and, for p < U, by the chunk's x loads.
// The last chunk loads its own x and weights once more (valid addresses, values unused) so that the counts hold.
template <int MT, int NT, int NLOC, int NW, int SPC, int NRT, int NSLOT, int U, int NBUF>
__global__ __launch_bounds__(64 * NW, (NW == 8 ? 2 : 1) * (3 - NBUF)) void lc_forward_direct_kernel(
    Geom g, const float *__restrict__ x, const float *__restrict__ w, const float *__restrict__ bias, float alpha,
    const float *__restrict__ alpha_dev, float *__restrict__ y, int strips_per_row, int sq4, int RV, int work_offset,
    int nbt) {
    typedef typename FVec<NT>::T WV;          // NT consecutive weights / outputs
    constexpr int BT = 16 * MT, NFW = NW / NLOC, NTHR = 64 * NW;
    constexpr int NS = SPC * NRT;             // k-steps per chunk
    constexpr int NG4 = SPC / 4, GT = SPC % 4, NG = NG4 + (GT ? 1 : 0);
    constexpr int BUF = NSLOT * NTHR * 4;     // floats per buffer
    static_assert(NS % U == 0 && U <= NS, "the weight ring turns a whole number of times per chunk");
    static_assert(U - 1 + NSLOT <= 63 && NS <= 63, "the memory counter has six bits");
    extern __shared__ __attribute__((aligned(16))) float xs[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, kk = lane >> 4;
    const int t_id = remap_xcd(blockIdx.x, gridDim.x);
    const int work = work_offset + t_id / nbt;
    const int i = work / strips_per_row, j0 = (work - i * strips_per_row) * NLOC;
    const int b0 = (t_id % nbt) * BT;
    const int wl = wave % NLOC, wf = wave / NLOC;
    const int j = j0 + wl;
    const int f0 = (blockIdx.y * NFW + wf) * NT * 16;
    const bool active = j < g.LW;
    const int loc = i * g.LW + (active ? j : g.LW - 1);   // idle waves shadow the last field of the row
    const int SC = g.S * g.C, WC = g.W * g.C, RS = RV * 4;
    const size_t img = (size_t)g.H * WC;
    const int col0 = j0 * SC;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int u = 0; u < NT; ++u) acc[mt][u] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // weights: w[loc] is K rows of F floats; the lane's part of the address is its row inside a group and its filters
    gbyte_ptr wloc = (gbyte_ptr)(w + (size_t)loc * g.K * g.F + f0);
    const unsigned wlane4 = (unsigned)((4 * kk * g.F + NT * n) * 4), wlaneT = (unsigned)((GT * kk * g.F + NT * n) * 4);
    // row of w[l], relative to the chunk's first, that k-step p of a chunk contracts for lanes kk = 0
    auto step_row = [&](int p) -> int {
        const int r = p / SPC, sidx = p - r * SPC, gi = sidx / 4;
        return r * g.RC + (gi < NG4 ? 16 * gi + (sidx & 3) : 16 * NG4 + (sidx - 4 * NG4));
    };
    auto step_lane = [&](int p) -> unsigned { return (p % SPC) / 4 < NG4 ? wlane4 : wlaneT; };
    auto wchunk = [&](int kh) -> gbyte_ptr { return wloc + (size_t)kh * g.RC * g.F * 4; };
    WV wr[U];
#pragma unroll
    for (int p = 0; p < U; ++p) wr[p] = load_nowait<NT>(wloc + (size_t)step_row(p) * g.F * 4, step_lane(p));

    // where this lane's vector of load q comes from: bytes past the chunk's first vector (image b0, image row
    // i*S + kh, column col0)
    unsigned goff[NSLOT];
    {
        const int lim = WC - col0 - 4;        // last float offset from col0 at which a whole vector is inside the row
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            const int P = q * NTHR + tid, b = P / RV, v = P - b * RV;
            const int r = v / sq4, vv = v - r * sq4;
            const bool data = b < BT && r < NRT;
            const int bc = min(b, g.B - 1 - b0);
            goff[q] = data ? (unsigned)(((size_t)bc * img + (size_t)r * WC + min(4 * vv, max(lim, 0))) * 4) : 0u;
        }
    }
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) float *)xs + wave * 64 * 16;
    auto stage = [&](int kh, int buf) {
        gbyte_ptr base = (gbyte_ptr)(x + (size_t)b0 * img + (size_t)(i * g.S + kh) * WC + col0);
        const unsigned l = lds0 + buf * (BUF * 4);
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) load_lds16(base, goff[q], l + q * (NTHR * 16));
    };
    // With two buffers and a ring as deep as a chunk, the x loads of the next chunk go out one or a few at a time
    // behind the MFMAs of the first half of the k-steps (SPS per step) instead of all at the chunk's start, where they
    // queue up in the compute unit's one address unit with the waves, which issue in order, standing behind them;
    // in the first half, so that the last one has half a chunk to land.
    constexpr bool kSpread = NBUF == 2 && U == NS;
    constexpr int NSP = NS / 2 > 0 ? NS / 2 : 1, SPS = (NSLOT + NSP - 1) / NSP;
    constexpr int kLastDmaStep = (NSLOT - 1) / SPS;
    auto dma_in_step = [&](int p) -> int {     // x loads issued in k-step p
        const int lo = p * SPS, hi = (p + 1) * SPS < NSLOT ? (p + 1) * SPS : NSLOT;
        return hi > lo ? hi - lo : 0;
    };

    // the lane's four floats of group gi, patch row r of the chunk, image m + 16 mt: abase + mt*16*RS + r*sq4*4 + 16 gi
    const float *abase = xs + (lane & 15) * RS + wl * SC + 4 * kk;
    const float *abaseT = xs + (lane & 15) * RS + wl * SC + 16 * NG4 + GT * kk;
    if constexpr (NBUF == 2) {
        stage(0, 0);
        wait_loads<0>();
        __syncthreads();
    }
    int c = 0;
    for (int kh = 0; kh < g.R; kh += NRT, ++c) {
        const int khn = kh + NRT < g.R ? kh + NRT : kh;       // the last chunk reloads itself
        const float *arow = abase, *arowT = abaseT;
        gbyte_ptr xnext = (gbyte_ptr)(x + (size_t)b0 * img + (size_t)(i * g.S + khn) * WC + col0);
        const unsigned lnext = lds0 + ((c + 1) & 1) * (BUF * 4);
        if constexpr (NBUF == 2) {
            if constexpr (!kSpread) stage(khn, (c + 1) & 1);
            arow += (c & 1) * BUF;
            arowT += (c & 1) * BUF;
        } else {
            if (c > 0) __syncthreads();      // everybody is through with the previous chunk
            stage(kh, 0);
            wait_loads<0>();
            __syncthreads();
        }
        gbyte_ptr wc = wchunk(kh), wn = wchunk(khn);
        // the lane's A operands of group gi of patch row r: four consecutive floats (8-byte aligned: two halves in
        // one LDS instruction), or the tail group's GT floats
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        float a[2][MT][4];
        auto read_group = [&](int r, int gi, float (&dst)[MT][4]) {
            if (gi < NG4) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const f32x2 lo = *(const f32x2 *)(arow + mt * 16 * RS + r * sq4 * 4 + 16 * gi);
                    const f32x2 hi = *(const f32x2 *)(arow + mt * 16 * RS + r * sq4 * 4 + 16 * gi + 2);
                    dst[mt][0] = lo[0]; dst[mt][1] = lo[1]; dst[mt][2] = hi[0]; dst[mt][3] = hi[1];
                }
            } else {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int t = 0; t < GT; ++t) dst[mt][t] = arowT[mt * 16 * RS + r * sq4 * 4 + t];
            }
        };
        read_group(0, 0, a[0]);
#pragma unroll
        for (int r = 0; r < NRT; ++r) {
#pragma unroll
            for (int gi = 0; gi < NG; ++gi) {
                const int G = gi < NG4 ? 4 : GT, cur = (r * NG + gi) & 1;
#pragma unroll
                for (int t = 0; t < G; ++t) {
                    const int p = r * SPC + 4 * gi + t;       // k-step of the chunk
                    // (the loop is unrolled: p is a constant by the time this is compiled)
                    if constexpr (kSpread) {
                        // behind the weights of k-step p: the other NS-1 weight loads and every x load but this step's own
                        wait_loads_minus<NS - 1 + NSLOT, SPS>(dma_in_step(p), wr[p % U]);
                    } else {
                        if (p < U) wait_loads<U - 1 + NSLOT>(wr[p % U]);
                        else wait_loads<U - 1>(wr[p % U]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int u = 0; u < NT; ++u)
                            acc[mt][u] = mfma16(a[cur][mt][t], fget<NT>(wr[p % U], u), acc[mt][u]);
                    __builtin_amdgcn_sched_barrier(0);
                    // behind the group's first MFMAs: the LDS reads of the next group
                    if (t == 0) {
                        if (gi + 1 < NG) read_group(r, gi + 1, a[cur ^ 1]);
                        else if (r + 1 < NRT) read_group(r + 1, 0, a[cur ^ 1]);
                    }
                    if constexpr (kSpread) {
#pragma unroll
                        for (int q = p * SPS; q < (p + 1) * SPS && q < NSLOT; ++q)
                            load_lds16(xnext, goff[q], lnext + q * (NTHR * 16));
                    }
                    const int pn = p + U;                     // the k-step whose weights take this ring slot
                    gbyte_ptr wp = pn < NS ? wc : wn;
                    const int pp = pn < NS ? pn : pn - NS;
                    wr[p % U] = load_nowait<NT>(wp + (size_t)step_row(pp) * g.F * 4, step_lane(pp));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        if constexpr (NBUF == 2) {
            // this lane's x loads of the next chunk have landed (the weight loads behind the last of them may fly on)
            if constexpr (kSpread) wait_loads<NS - kLastDmaStep>();
            else wait_loads<NS>();
            __syncthreads();
        }
    }
    // the weights loaded last are not used: they must have landed before their registers are given up
#pragma unroll
    for (int p = 0; p < U; ++p) wait_loads<0>(wr[p]);

    if (!active) return;
    if (alpha_dev) alpha = *alpha_dev;
    WV bv;
    if constexpr (NT == 1) bv = 0.f; else bv = (WV)(0.f);
    if (bias) bv = *(const WV *)(bias + (size_t)loc * g.F + f0 + NT * n);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int b = b0 + mt * 16 + 4 * kk + r;
            if (b >= g.B) continue;
            WV o;
            if constexpr (NT == 1) {
                o = alpha * acc[mt][0][r] + bv;
            } else {
#pragma unroll
                for (int u = 0; u < NT; ++u) o[u] = alpha * acc[mt][u][r] + bv[u];
            }
            *(WV *)(y + ((size_t)b * g.L + loc) * g.F + f0 + NT * n) = o;
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

// Host check of a lc_forward_kernel launch.  tparam = {MT, NT, NLOC, bytes per operand element}; arg = {strips per field row, staged floats
// per image (sq), LDS row stride (rs)}.  The kernel masks every ragged edge itself, so what has to hold is that
// the grid covers (strip, filter block, batch tile) and that a staged strip row fits its LDS row.
int check_forward_generic(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0], NT = p.tparam[1], NLOC = p.tparam[2];
    const int strips = p.arg[0], sq = p.arg[1], rs = p.arg[2];
    const int BT = 16 * MT, NFW = 4 / NLOC;
    LC_PLAN_REQUIRE(p, NLOC == 1 || NLOC == 2 || NLOC == 4);
    LC_PLAN_REQUIRE(p, p.block == 256);
    LC_PLAN_REQUIRE(p, strips == ceil_div(g.LW, NLOC) && (long long)p.grid[0] == (long long)strips * g.LH);
    LC_PLAN_REQUIRE(p, (long long)p.grid[1] * NFW * NT * 16 >= g.F && (long long)(p.grid[1] - 1) * NFW * NT * 16 < g.F);
    LC_PLAN_REQUIRE(p, (long long)p.grid[2] * BT >= g.B && (long long)(p.grid[2] - 1) * BT < g.B);
    LC_PLAN_REQUIRE(p, sq == (g.R + (NLOC - 1) * g.S) * g.C);
    // a wave reads up to 3 floats past its window's last whole 4-element step
    LC_PLAN_REQUIRE(p, rs >= sq + 3);
    LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)BT * rs * sizeof(float));
    return LC_OK;
}

template <int MT, int NT, int NLOC, typename T>
int launch_one(const Geom &g, const T *x, const T *w, const float *bias, float alpha,
               const float *alpha_dev, float *y, hipStream_t s) {
    constexpr int BT = 16 * MT, NFW = 4 / NLOC;
    const int strips = (g.LW + NLOC - 1) / NLOC;
    const int sq = (g.R + (NLOC - 1) * g.S) * g.C;
    const int rs = lds_row_stride(sq);
    const size_t lds = ((size_t)BT * rs + 8) * sizeof(float);
    if (lds > 160 * 1024) return LC_EUNSUPPORTED;
    auto kern = lc_forward_kernel<MT, NT, NLOC, T>;
    dim3 grid(strips * g.LH, (g.F + NFW * NT * 16 - 1) / (NFW * NT * 16), (g.B + BT - 1) / BT);
    const LaunchPlan plan = make_plan("lc_forward_generic", {MT, NT, NLOC, (int)sizeof(T)}, {strips, sq, rs}, grid, 256, lds);
    if (int rc = check_forward_generic(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_forward launch", kern, s, g, x, w, bias, alpha, alpha_dev, y, strips, sq, rs);
    return LC_OK;
}

}  // namespace

namespace {

int fast_row_stride(int sqc) {
    // stride == 4 (mod 32) floats: the 16 images x 4 k-offsets a wave reads per A operand spread over the banks
    return ((sqc + 31) / 32) * 32 + 4;
}

// Host check of a lc_forward_fast_kernel launch.
// tparam = {MT, NT, NLOC, UNR, NW, bytes per operand element, SPC, NRT, staging slots per lane};
// arg = {CQ, sq4, RS, NR, first strip, strips in this launch, batch tiles, strips per field row}.
int check_forward_fast(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0], NT = p.tparam[1], NLOC = p.tparam[2], UNR = p.tparam[3], NW = p.tparam[4];
    const int ES = p.tparam[5], SPC = p.tparam[6], NRT = p.tparam[7], SLOTS = p.tparam[8];
    const int CQ = p.arg[0], sq4 = p.arg[1], RS = p.arg[2], NR = p.arg[3], first = p.arg[4], count = p.arg[5];
    const int nbt = p.arg[6], strips = p.arg[7];
    LC_PLAN_REQUIRE(p, NLOC > 0 && NW % NLOC == 0 && (ES == 4 || ES == 2) && (NT == 1 || NT == 2 || NT == 4));
    const int BT = 16 * MT, NFW = NW / NLOC, NTHR = 64 * NW, SC = g.S * g.C, WC = g.W * g.C, sqc = 4 * sq4;
    LC_PLAN_REQUIRE(p, (int)p.block == NTHR);
    // four-element vector accesses: patch rows, image rows and strip starts in whole vectors
    LC_PLAN_REQUIRE(p, g.RC % 4 == 0 && WC % 4 == 0 && (NLOC * SC) % 4 == 0);
    // filters in whole tiles, every block of filters exactly once
    LC_PLAN_REQUIRE(p, g.F % (NFW * NT * 16) == 0 && (int)p.grid[1] == g.F / (NFW * NT * 16) && p.grid[2] == 1);
    // the contraction: chunks of CQ floats of a patch row in ring turns of UNR k-steps; several patch rows per chunk
    // only as whole rows
    LC_PLAN_REQUIRE(p, CQ > 0 && CQ % (4 * UNR) == 0 && g.RC % CQ == 0);
    LC_PLAN_REQUIRE(p, NR >= 1 && NR <= 15 && g.R % NR == 0 && (NR == 1 || CQ == g.RC));
    LC_PLAN_REQUIRE(p, g.K / 4 >= UNR);
    // the staged strip: covers every field's window, fits the packed slot index, the staging registers and its LDS row
    LC_PLAN_REQUIRE(p, sqc >= CQ + (NLOC - 1) * SC && sqc <= 4096 && BT <= 0x3fff);
    LC_PLAN_REQUIRE(p, (long long)BT * NR * sq4 <= (long long)SLOTS * NTHR);
    LC_PLAN_REQUIRE(p, RS % 2 == 0 && RS >= NR * sqc + 2);
    LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)BT * RS * sizeof(float));
    // the strips of this launch, each with every batch tile
    LC_PLAN_REQUIRE(p, strips == ceil_div(g.LW, NLOC) && nbt == ceil_div(g.B, BT));
    LC_PLAN_REQUIRE(p, first >= 0 && count >= 1 && first + count <= strips * g.LH);
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] == (long long)count * nbt);
    if (SPC > 0) {
        // compile-time counts: one chunk = NRT whole patch rows of SPC k-steps, fp32 only, 32-bit staging offsets;
        // every slot loads from an address clamped into the image, which needs four floats from every strip's start
        LC_PLAN_REQUIRE(p, ES == 4 && CQ == g.RC && SPC == CQ / 4 && NRT == NR && SPC % UNR == 0);
        LC_PLAN_REQUIRE(p, (long long)g.B * g.H * g.W * g.C < (1LL << 31));
        LC_PLAN_REQUIRE(p, WC - (strips - 1) * NLOC * SC >= 4);
    } else {
        LC_PLAN_REQUIRE(p, NRT == 1);
    }
    return LC_OK;
}

template <int MT, int NT, int NLOC, int UNR, int NW = 4, int SPC = 0, int NRT = 1, int NSL = 0, typename T>
int launch_fast(const Geom &g, const T *x, const T *w, const float *bias, float alpha,
                const float *alpha_dev, float *y, int CQ, int NR, int work_first, int work_count, hipStream_t s) {
    constexpr int BT = 16 * MT, NFW = NW / NLOC;
    constexpr int SLOTS = NSL > 0 ? NSL : (NW == 8 ? kFwdStageSlotsWide : kFwdStageSlots);   // as in the kernel
    const int sqc = (CQ + (NLOC - 1) * g.S * g.C + 3) & ~3;   // staged floats per image and patch row
    const int RS = fast_row_stride(NR * sqc);
    const size_t lds = (size_t)BT * RS * sizeof(float);
    auto kern = lc_forward_fast_kernel<MT, NT, NLOC, UNR, NW, T, SPC, NRT, NSL>;
    const int strips = (g.LW + NLOC - 1) / NLOC;
    const int nbt = (g.B + BT - 1) / BT;
    dim3 grid(work_count * nbt, g.F / (NFW * NT * 16));
    const LaunchPlan plan = make_plan("lc_forward_fast", {MT, NT, NLOC, UNR, NW, (int)sizeof(T), SPC, NRT, SLOTS},
                                      {CQ, sqc / 4, RS, NR, work_first, work_count, nbt, strips}, grid, 64 * NW, lds);
    if (int rc = check_forward_fast(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_forward launch", kern, s, g, x, w, bias, alpha, alpha_dev, y, strips, CQ, sqc / 4, RS, NR,
              work_first, nbt);
    return LC_OK;
}

// Host check of a lc_forward_direct_kernel launch.
// tparam = {MT, NT, NLOC, U (weight ring, k-steps), NW, 4, SPC, NRT, NSLOT (x loads per lane and chunk), NBUF};
// arg = {RC, sq4, LDS row stride in floats, NRT, first strip, strips in this launch, batch tiles, strips per field row}.
int check_forward_direct(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0], NT = p.tparam[1], NLOC = p.tparam[2], U = p.tparam[3], NW = p.tparam[4];
    const int SPC = p.tparam[6], NRT = p.tparam[7], NSLOT = p.tparam[8], NBUF = p.tparam[9];
    const int sq4 = p.arg[1], RS = p.arg[2], first = p.arg[4], count = p.arg[5], nbt = p.arg[6], strips = p.arg[7];
    LC_PLAN_REQUIRE(p, NLOC > 0 && NW % NLOC == 0 && (NT == 1 || NT == 2 || NT == 4) && (NBUF == 1 || NBUF == 2));
    const int BT = 16 * MT, NFW = NW / NLOC, NTHR = 64 * NW, SC = g.S * g.C, WC = g.W * g.C, NS = SPC * NRT;
    LC_PLAN_REQUIRE(p, (int)p.block == NTHR && p.arg[0] == g.RC && p.arg[3] == NRT);
    // whole patch rows of SPC k-steps, NRT of them per chunk; 16-byte vectors of x from every strip's start; the
    // 8-byte LDS reads of a field's window
    LC_PLAN_REQUIRE(p, g.RC == 4 * SPC && NRT >= 1 && g.R % NRT == 0 && WC % 4 == 0 && (NLOC * SC) % 4 == 0 && SC % 2 == 0);
    LC_PLAN_REQUIRE(p, g.F % (NFW * NT * 16) == 0 && (int)p.grid[1] == g.F / (NFW * NT * 16) && p.grid[2] == 1);
    // the staged strip covers every field's window; an LDS row is NRT pieces of sq4 vectors, an odd number of vectors
    LC_PLAN_REQUIRE(p, 4 * sq4 >= g.RC + (NLOC - 1) * SC && RS % 4 == 0 && RS / 4 >= NRT * sq4 && (RS / 4) % 2 == 1);
    LC_PLAN_REQUIRE(p, (long long)NSLOT * NTHR >= (long long)BT * (RS / 4));
    LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)NBUF * NSLOT * NTHR * 16);
    // the waits in the kernel count the loads in flight (a six-bit counter); the ring turns whole times per chunk
    LC_PLAN_REQUIRE(p, U >= 1 && U <= NS && NS % U == 0 && U - 1 + NSLOT <= 63 && NS <= 63);
    // 32-bit byte offsets into x; clamped vectors stay inside the image row
    LC_PLAN_REQUIRE(p, (long long)g.B * g.H * g.W * g.C * 4 < (1LL << 32));
    LC_PLAN_REQUIRE(p, strips == ceil_div(g.LW, NLOC) && nbt == ceil_div(g.B, BT));
    LC_PLAN_REQUIRE(p, WC - (strips - 1) * NLOC * SC >= 4);
    LC_PLAN_REQUIRE(p, first >= 0 && count >= 1 && first + count <= strips * g.LH);
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] == (long long)count * nbt);
    return LC_OK;
}

// whether lc_forward_direct_kernel<.., SPC, NRT, NSLOT, ..> takes the layer (fp32 operands)
template <int MT, int NLOC, int NW, int SPC, int NRT, int NSLOT>
bool forward_direct_fits(const Geom &g) {
    const int SC = g.S * g.C, WC = g.W * g.C, strips = (g.LW + NLOC - 1) / NLOC;
    const int sq4 = ((g.RC + (NLOC - 1) * SC + 3) & ~3) / 4, RV = (NRT * sq4) | 1;
    return g.RC == 4 * SPC && g.R % NRT == 0 && WC % 4 == 0 && (NLOC * SC) % 4 == 0 && SC % 2 == 0 &&
           (16 * MT * RV + 64 * NW - 1) / (64 * NW) == NSLOT && (long long)g.B * g.H * g.W * g.C * 4 < (1LL << 32) &&
           WC - (strips - 1) * NLOC * SC >= 4;
}

template <int MT, int NT, int NLOC, int NW, int SPC, int NRT, int NSLOT, int U, int NBUF>
int launch_direct(const Geom &g, const float *x, const float *w, const float *bias, float alpha,
                  const float *alpha_dev, float *y, int work_first, int work_count, hipStream_t s) {
    constexpr int BT = 16 * MT, NFW = NW / NLOC, NTHR = 64 * NW;
    const int sq4 = ((g.RC + (NLOC - 1) * g.S * g.C + 3) & ~3) / 4, RV = (NRT * sq4) | 1;
    const size_t lds = (size_t)NBUF * NSLOT * NTHR * 16;
    auto kern = lc_forward_direct_kernel<MT, NT, NLOC, NW, SPC, NRT, NSLOT, U, NBUF>;
    const int strips = (g.LW + NLOC - 1) / NLOC;
    const int nbt = (g.B + BT - 1) / BT;
    dim3 grid(work_count * nbt, g.F / (NFW * NT * 16));
    const LaunchPlan plan = make_plan("lc_forward_direct", {MT, NT, NLOC, U, NW, 4, SPC, NRT, NSLOT, NBUF},
                                      {g.RC, sq4, RV * 4, NRT, work_first, work_count, nbt, strips}, grid, NTHR, lds);
    if (int rc = check_forward_direct(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_forward launch", kern, s, g, x, w, bias, alpha, alpha_dev, y, strips, sq4, RV, work_first, nbt);
    return LC_OK;
}

// Workgroups of the big tile are long (a strip of fields times the whole batch tile) and only two fit a
// compute unit, so a grid that is not a multiple of 2 x 256 ends in a round that leaves most of the
// chip idle.  The strips of that last partial round are therefore issued as a second launch whose
// workgroups take a quarter of the batch tile each: four times as many, a quarter as long.
constexpr int kComputeUnits = 256, kBigTilesPerCu = 2;

template <int MT, int NT, int NLOC, int UNR, typename T>
int launch_fast_tiered(const Geom &g, const T *x, const T *w, const float *bias, float alpha,
                       const float *alpha_dev, float *y, int CQ, hipStream_t s) {
    const int strips = (g.LW + NLOC - 1) / NLOC;
    const int ntask = strips * g.LH, slots = kComputeUnits * kBigTilesPerCu;
    const int zb = (g.B + 16 * MT - 1) / (16 * MT) * (g.F / ((4 / NLOC) * NT * 16));
    const int rounds = (ntask * zb) / slots, rem = ntask * zb - rounds * slots;
    if constexpr (MT == 8) {
        if (zb == 1 && rounds >= 1 && rounds <= 6 && rem > 0 && rem <= slots / 4) {
            const int first = rounds * slots;
            // whole patch rows of 15 k-steps that fill every staging slot: the variant with compile-time counts
            const int sqc = (CQ + (NLOC - 1) * g.S * g.C + 3) & ~3;
            const bool fixed = UNR == 5 && sizeof(T) == 4 && CQ == g.RC && (CQ >> 2) == 15 &&
                               (16 * MT * (sqc / 4) + 255) / 256 == kFwdStageSlots &&
                               (long long)g.B * g.H * g.W * g.C < (1LL << 31);
            int rc = fixed ? launch_fast<MT, NT, NLOC, UNR, 4, 15>(g, x, w, bias, alpha, alpha_dev, y, CQ, 1, 0, first, s)
                           : launch_fast<MT, NT, NLOC, UNR>(g, x, w, bias, alpha, alpha_dev, y, CQ, 1, 0, first, s);
            if (rc != LC_OK) return rc;
            // the short workgroups stage four patch rows at a time (same LDS footprint as the long ones),
            // so that a chunk's MFMAs still cover the latency of fetching the next one
            int nr = 1;
            if (CQ == g.RC) {
                for (int c : {4, 3, 2})
                    if (g.R % c == 0) { nr = c; break; }
            }
            // their k-steps are short (2 x NT MFMAs), so the weight ring is made as deep as a whole patch row;
            // four whole rows of 15 k-steps that fill every staging slot: the variant with compile-time counts
            if ((CQ >> 2) == 15 && fixed && nr == 4 && 32 * 4 * (sqc / 4) == kFwdStageSlots * 256)
                return launch_fast<2, NT, NLOC, 15, 4, 15, 4>(g, x, w, bias, alpha, alpha_dev, y, CQ, nr, first, ntask - first, s);
            if ((CQ >> 2) % 15 == 0)
                return launch_fast<2, NT, NLOC, 15>(g, x, w, bias, alpha, alpha_dev, y, CQ, nr, first, ntask - first, s);
            if ((CQ >> 2) % 16 == 0)
                return launch_fast<2, NT, NLOC, 16>(g, x, w, bias, alpha, alpha_dev, y, CQ, nr, first, ntask - first, s);
            return launch_fast<2, NT, NLOC, UNR>(g, x, w, bias, alpha, alpha_dev, y, CQ, nr, first, ntask - first, s);
        }
    }
    // 32-image tiles (small layers) are latency-bound: several patch rows per chunk halve the barriers and let
    // more loads fly at once, as far as the staging registers and the LDS budget allow
    int nr = 1;
    if constexpr (MT <= 2) {
        if (CQ == g.RC) {
            const int sqc = (CQ + (NLOC - 1) * g.S * g.C + 3) & ~3;
            for (int c : {4, 3, 2})
                if (g.R % c == 0 && (size_t)16 * MT * c * (sqc / 4) <= (size_t)kFwdStageSlots * 256 &&
                    (size_t)16 * MT * fast_row_stride(c * sqc) * 4 <= 52 * 1024 && c <= 15) { nr = c; break; }
        }
    }
    // 32-image tiles, two patch rows of 12 k-steps in eight staging slots: compile-time counts
    if constexpr (MT == 2 && UNR == 6 && sizeof(T) == 4) {
        const int sq4 = ((CQ + (NLOC - 1) * g.S * g.C + 3) & ~3) / 4;
        if (CQ == g.RC && (CQ >> 2) == 12 && nr == 2 && g.R % 2 == 0 && (32 * 2 * sq4 + 255) / 256 == 8 &&
            (long long)g.B * g.H * g.W * g.C < (1LL << 31))
            return launch_fast<MT, NT, NLOC, UNR, 4, 12, 2, 8>(g, x, w, bias, alpha, alpha_dev, y, CQ, nr, 0, ntask, s);
    }
    // 32-image tiles whose chunks (whole patch rows) fill every staging slot: the variants with compile-time counts
    if constexpr (MT == 2 && UNR == 8 && sizeof(T) == 4) {
        const int sq4 = ((CQ + (NLOC - 1) * g.S * g.C + 3) & ~3) / 4;
        const bool fits = CQ == g.RC && 32 * nr * sq4 == kFwdStageSlots * 256 && g.R % nr == 0 &&
                          (long long)g.B * g.H * g.W * g.C < (1LL << 31);
        if (fits && (CQ >> 2) == 24 && nr == 2)
            return launch_fast<MT, NT, NLOC, UNR, 4, 24, 2>(g, x, w, bias, alpha, alpha_dev, y, CQ, nr, 0, ntask, s);
        if (fits && (CQ >> 2) == 48 && nr == 1)
            return launch_fast<MT, NT, NLOC, UNR, 4, 48, 1>(g, x, w, bias, alpha, alpha_dev, y, CQ, nr, 0, ntask, s);
    }
    return launch_fast<MT, NT, NLOC, UNR>(g, x, w, bias, alpha, alpha_dev, y, CQ, nr, 0, ntask, s);
}

// Picks the chunk (CQ floats of a patch row, a divisor of RC and multiple of 4*UNR) so that the staged
// strip of BT images fits the staging registers and the LDS budget.  Returns 0 if none does.
int pick_chunk(const Geom &g, int BT, int NLOC, int UNR, size_t lds_budget, int nthr = 256,
               int slots = kFwdStageSlots) {
    const int SC = g.S * g.C;
    for (int nsub = 1; nsub <= g.RC / (4 * UNR); ++nsub) {
        if (g.RC % nsub) continue;
        const int CQ = g.RC / nsub;
        if (CQ % (4 * UNR)) continue;
        const int sqc = (CQ + (NLOC - 1) * SC + 3) & ~3;
        if ((size_t)BT * (sqc / 4) > (size_t)slots * nthr) continue;
        if ((size_t)BT * fast_row_stride(sqc) * 4 > lds_budget) continue;
        if (sqc / 4 > 0xffff / 4) continue;
        return CQ;
    }
    return 0;
}

template <int MT, int NT, int NLOC, typename T>
int launch_fast_unr(const Geom &g, const T *x, const T *w, const float *bias, float alpha,
                    const float *alpha_dev, float *y, hipStream_t s, bool *done) {
    const size_t budget = 52 * 1024;  // three workgroups per compute unit
    *done = true;
    const int spr = g.RC / 4;
    int CQ;
    if (spr % 8 == 0 && (CQ = pick_chunk(g, 16 * MT, NLOC, 8, budget)))
        return launch_fast_tiered<MT, NT, NLOC, 8>(g, x, w, bias, alpha, alpha_dev, y, CQ, s);
    if (spr % 6 == 0 && (CQ = pick_chunk(g, 16 * MT, NLOC, 6, budget)))
        return launch_fast_tiered<MT, NT, NLOC, 6>(g, x, w, bias, alpha, alpha_dev, y, CQ, s);
    if (spr % 5 == 0 && (CQ = pick_chunk(g, 16 * MT, NLOC, 5, budget)))
        return launch_fast_tiered<MT, NT, NLOC, 5>(g, x, w, bias, alpha, alpha_dev, y, CQ, s);
    *done = false;
    return LC_OK;
}

// Layers with 16 filters per field give a wave one filter tile, so a staged strip feeds few MFMAs.  Eight
// waves (eight fields) per workgroup share a strip that is only about a third longer than the one four
// fields need, and with so few accumulators two such workgroups still fit a compute unit.
template <typename T>
int launch_fast_wide(const Geom &g, const T *x, const T *w, const float *bias, float alpha,
                     const float *alpha_dev, float *y, hipStream_t s, bool *done) {
    const size_t budget = 78 * 1024;
    const int spr = g.RC / 4, ntask = ((g.LW + 7) / 8) * g.LH;
    *done = true;
    int CQ;
    if (spr % 8 == 0 && (CQ = pick_chunk(g, 128, 8, 8, budget, 512, kFwdStageSlotsWide)))
        return launch_fast<8, 1, 8, 8, 8>(g, x, w, bias, alpha, alpha_dev, y, CQ, 1, 0, ntask, s);
    if (spr % 6 == 0 && (CQ = pick_chunk(g, 128, 8, 6, budget, 512, kFwdStageSlotsWide))) {
        // whole patch rows of 12 k-steps that need every staging slot: the variant with compile-time counts
        const int sq4 = ((CQ + 7 * g.S * g.C + 3) & ~3) / 4;
        if constexpr (sizeof(T) == 4) {
            // sixteen fields per workgroup (four waves per SIMD) where that idles no more waves at the end of a field
            // row than eight do: the per-chunk costs that do not shrink with the chunk (barrier, first LDS reads) are
            // spread over twice the MFMAs (57 fields per row, 128 x 128 x 3 input: 121 -> 107 us)
            if ((g.LW + 15) / 16 * 2 == (g.LW + 7) / 8 && forward_direct_fits<8, 16, 16, 12, 1, 5>(g))
                return launch_direct<8, 1, 16, 16, 12, 1, 5, 12, 2>(g, x, w, bias, alpha, alpha_dev, y, 0,
                                                                    ((g.LW + 15) / 16) * g.LH, s);
            if (forward_direct_fits<8, 8, 8, 12, 1, 6>(g))
                return launch_direct<8, 1, 8, 8, 12, 1, 6, 12, 2>(g, x, w, bias, alpha, alpha_dev, y, 0, ntask, s);
        }
        if (sizeof(T) == 4 && CQ == g.RC && spr == 12 && (128 * sq4 + 511) / 512 == kFwdStageSlotsWide &&
            (long long)g.B * g.H * g.W * g.C < (1LL << 31))
            return launch_fast<8, 1, 8, 6, 8, 12>(g, x, w, bias, alpha, alpha_dev, y, CQ, 1, 0, ntask, s);
        return launch_fast<8, 1, 8, 6, 8>(g, x, w, bias, alpha, alpha_dev, y, CQ, 1, 0, ntask, s);
    }
    if (spr % 5 == 0 && (CQ = pick_chunk(g, 128, 8, 5, budget, 512, kFwdStageSlotsWide)))
        return launch_fast<8, 1, 8, 5, 8>(g, x, w, bias, alpha, alpha_dev, y, CQ, 1, 0, ntask, s);
    *done = false;
    return LC_OK;
}

// filters per wave / fields per workgroup by F (at most nt_cap tiles of 16 filters per wave)
template <int MT, typename T>
int launch_fast_mt(const Geom &g, const T *x, const T *w, const float *bias, float alpha,
                   const float *alpha_dev, float *y, hipStream_t s, bool *done, int nt_cap) {
    *done = false;
    if (g.F % 128 == 0 && nt_cap >= 4) return launch_fast_unr<MT, 4, 2>(g, x, w, bias, alpha, alpha_dev, y, s, done);
    if (g.F % 64 == 0 && nt_cap >= 4) return launch_fast_unr<MT, 4, 4>(g, x, w, bias, alpha, alpha_dev, y, s, done);
    if (g.F % 32 == 0 && nt_cap >= 2) return launch_fast_unr<MT, 2, 4>(g, x, w, bias, alpha, alpha_dev, y, s, done);
    if (g.F % 16 == 0) return launch_fast_unr<MT, 1, 4>(g, x, w, bias, alpha, alpha_dev, y, s, done);
    return LC_OK;
}

// workgroups of the pipelined kernel for a wave tile of 16*mt images x 16*nt filters
long long fast_workgroups(const Geom &g, int mt, int nt) {
    const int ntf = g.F % 128 == 0 && nt >= 4 ? 4 : g.F % 64 == 0 && nt >= 4 ? 4 : g.F % 32 == 0 && nt >= 2 ? 2 : 1;
    const int nloc = g.F % 128 == 0 && nt >= 4 ? 2 : 4;
    const long long strips = (g.LW + nloc - 1) / nloc;
    return strips * g.LH * ((g.B + 16 * mt - 1) / (16 * mt)) * (g.F / ((4 / nloc) * ntf * 16));
}

// The pipelined kernel for aligned shapes: patch rows that are whole 4-element runs, strips that start on a
// 4-element boundary (4 fields x S x C elements, or 2 when 128 filters are split over the waves).  *done_out tells
// whether a kernel was launched.
template <typename T>
int launch_forward_fast_path(const Geom &g, const T *x, const T *w, const float *bias, float alpha,
                             const float *alpha_dev, float *y, hipStream_t s, bool *done_out) {
    *done_out = false;
    const int nloc = g.F % 128 == 0 ? 2 : 4;
    const bool aligned = g.RC % 4 == 0 && (nloc * g.S * g.C) % 4 == 0 && (g.W * g.C) % 4 == 0 && g.K / 4 >= 16;
    // fp32, filters in blocks of 32, patch rows of 15 k-steps, at least one round of workgroups: the kernel that loads
    // x straight into LDS, on 64-image tiles (two buffers of a four-field strip, two workgroups per compute unit)
    // with a weight ring as deep as a whole patch row.  The strips that do not fill a last whole round of
    // 2 x 256 workgroups go out as a second launch of 32-image tiles.  (200 x 200 x 3 input, 46 x 46 fields of
    // 20 x 20, 32 filters, batch 128: 186 us against the 213 us of the 128-image tiles staged through registers;
    // ring depths of 5 k-steps: 205 us; 128-image tiles in this kernel: 257 us with one buffer, 274 us with two.)
    if constexpr (sizeof(T) == 4) {
        if (g.B > 64 && g.F % 32 == 0 && g.F % 64 != 0 && forward_direct_fits<4, 4, 4, 15, 1, 7>(g) &&
            forward_direct_fits<2, 4, 4, 15, 1, 4>(g)) {
            const int ntask = ((g.LW + 3) / 4) * g.LH, nbt = (g.B + 63) / 64, fy = g.F / 32;
            const long long per_strip = (long long)nbt * fy, slots = kComputeUnits * kBigTilesPerCu;
            if (ntask * per_strip >= slots) {
                const int first = (int)(ntask * per_strip / slots * slots / per_strip);
                *done_out = true;
                if (int rc = launch_direct<4, 2, 4, 4, 15, 1, 7, 15, 2>(g, x, w, bias, alpha, alpha_dev, y, 0, first, s))
                    return rc;
                if (first == ntask) return LC_OK;
                // (the rest on 16-image tiles instead, 320 workgroups: 189 against 187 us; LDS buffers cut down to the
                // rows themselves, 51 KB instead of 56, so that three workgroups of the main launch fit a compute
                // unit, with rounds of 3 x 256 workgroups: 185 us, and as one launch of all strips 189 us)
                return launch_direct<2, 2, 4, 4, 15, 1, 4, 15, 2>(g, x, w, bias, alpha, alpha_dev, y, first,
                                                                 ntask - first, s);
            }
        }
        // the same kernel on smaller layers of 32 filters, again with a ring as deep as the patch row: patch rows of
        // 24 k-steps on 32-image tiles where those give a round of workgroups (55 x 55 x 16 input, 6 x 6 fields at
        // stride 2, batch 128: 41.5 -> 34.5 us; a ring of 8 k-steps: 36.0 us), patch rows of 48 k-steps on 16-image
        // tiles and one filter tile per wave where even 32-image tiles give less than a round (23 x 23 x 32 input,
        // 81 fields: 23.4 -> 16.4 us; 32-image tiles 18.5 us)
        if (g.F % 32 == 0 && g.F % 64 != 0) {
            const int ntask = ((g.LW + 3) / 4) * g.LH;
            if (g.B > 32 && forward_direct_fits<2, 4, 4, 24, 1, 7>(g) &&
                (long long)ntask * ((g.B + 31) / 32) * (g.F / 32) >= kComputeUnits * kBigTilesPerCu) {
                *done_out = true;
                return launch_direct<2, 2, 4, 4, 24, 1, 7, 24, 2>(g, x, w, bias, alpha, alpha_dev, y, 0, ntask, s);
            }
            if (g.B > 16 && forward_direct_fits<1, 4, 4, 48, 1, 7>(g) &&
                (long long)ntask * ((g.B + 31) / 32) * (g.F / 16) < kComputeUnits * kBigTilesPerCu) {
                *done_out = true;
                return launch_direct<1, 1, 4, 4, 48, 1, 7, 48, 2>(g, x, w, bias, alpha, alpha_dev, y, 0, ntask, s);
            }
        }
    }
    if constexpr (sizeof(T) == 4) {
        // Wide layers (filters in blocks of 128) whose patch row is 12 k-steps, the paper's
        // first layer among them (Sec. 5: 16x16x3 patches): the LDS-direct kernel on 64-image
        // tiles with the whole patch row's weights in flight.  Measured on that layer at
        // batch 192: 4.69 ms against 5.03 ms for the register-staged kernel (80 % against
        // 74 % of the fp32 MFMA peak); a ring half as deep gives the same, two patch rows
        // per LDS round 4.73 ms.
        // Only where its workgroups (a pair of fields x 64 images x 128 filters) fill two rounds of the chip:
        // smaller layers keep the register-staged kernel, which steps down to smaller tiles.
        const long long wide_wgs = (long long)((g.LW + 1) / 2) * g.LH * ((g.B + 63) / 64) * (g.F / 128);
        if (g.F % 128 == 0 && g.B > 32 && wide_wgs >= 2 * kComputeUnits * kBigTilesPerCu &&
            forward_direct_fits<4, 2, 4, 12, 1, 4>(g)) {
            *done_out = true;
            return launch_direct<4, 4, 2, 4, 12, 1, 4, 12, 2>(g, x, w, bias, alpha, alpha_dev, y, 0,
                                                              ((g.LW + 1) / 2) * g.LH, s);
        }
    }
    if (aligned && g.B > 16) {
        bool done = false;
        int rc = LC_OK;
        // 128 images x 64 filters per wave would need 128 accumulator registers and leave room for one wave
        // per SIMD only: wide layers take the 64-image tile (two waves per SIMD; the second batch tile of a
        // strip finds the weights in L2).  A layer too small to fill one round of two workgroups per CU at that
        // tile size steps down to smaller wave tiles until it does: finer workgroups spread evenly over the CUs.
        int mt = g.B > 64 && g.F % 64 != 0 ? 8 : g.B > 32 ? 4 : 2, nt = 4;
        // (larger tiles with fewer workgroups measured slower: a 55 x 55 x 16 input under 6 x 6 fields at stride 2,
        // 32 filters, batch 128: 53 us with 64-image tiles and 350 workgroups against 42 us with 32-image tiles and 700)
        // and 16-image tiles for layers that stay under that count even at 32 images measured no better: 27.4 against
        // 28.5 us on a 96 x 96 x 3 input under 11 x 11 fields of 64 filters, 26.1 against 23.4 us on 81 fields of 32)
        while (fast_workgroups(g, mt, nt) < kComputeUnits * kBigTilesPerCu && (mt > 2 || nt > 1)) {
            if (nt > 1 && (nt >= mt || mt == 2)) nt >>= 1; else mt >>= 1;
        }
        // the eight-wave kernel's grid covers F in whole tiles of 16 filters; other F take the masked kernel below
        const bool one_tile = g.F % 16 == 0 && (g.F % 32 != 0 || nt == 1);
        if (mt == 8 && one_tile && g.LW >= 8 && (8 * g.S * g.C) % 4 == 0)
            rc = launch_fast_wide(g, x, w, bias, alpha, alpha_dev, y, s, &done);
        if (!done && mt == 8) rc = launch_fast_mt<8>(g, x, w, bias, alpha, alpha_dev, y, s, &done, nt);
        if (!done && mt >= 4 && g.B > 32) rc = launch_fast_mt<4>(g, x, w, bias, alpha, alpha_dev, y, s, &done, nt);
        if (!done) rc = launch_fast_mt<2>(g, x, w, bias, alpha, alpha_dev, y, s, &done, nt);
        *done_out = done;
        return rc;
    }
    return LC_OK;
}

}  // namespace

namespace {

// The masked kernel (any shape).  Picks the tile: as many images per wave as the batch offers (weights are re-read
// once per batch tile), then as many filters as fit the accumulator budget, then the widest strip that fits LDS.
template <typename T>
int launch_forward_generic(const Geom &g, const T *x, const T *w, const float *bias, float alpha,
                           const float *alpha_dev, float *y, hipStream_t s) {
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

}  // namespace

int launch_forward_f32(const Geom &g, const float *x, const float *w, const float *bias, float alpha,
                       const float *alpha_dev, float *y, hipStream_t s, void *ws, size_t ws_bytes) {
    // layers with 128-filter blocks: one field per workgroup, patches through LDS, 128 x 128 output tiles
    if (forward_wide_supported(g)) return launch_forward_wide_f32(g, x, w, bias, alpha, alpha_dev, y, ws, ws_bytes, s);
    // aligned shapes take the pipelined kernel: patch rows that are whole dwordx4 runs, strips that start on a
    // 16-byte boundary (4 fields x S x C floats, or 2 when 128 filters are split over the waves)
    {
        bool done = false;
        const int rc = launch_forward_fast_path(g, x, w, bias, alpha, alpha_dev, y, s, &done);
        if (done) return rc;
    }
    return launch_forward_generic(g, x, w, bias, alpha, alpha_dev, y, s);
}

int launch_forward_bf16_storage(const Geom &g, const void *x, const void *w, const float *bias, float alpha, float *y,
                                hipStream_t s) {
    bool done = false;
    const int rc = launch_forward_fast_path(g, (const bf16_t *)x, (const bf16_t *)w, bias, alpha, nullptr, y, s, &done);
    if (done) return rc;
    return launch_forward_generic(g, (const bf16_t *)x, (const bf16_t *)w, bias, alpha, nullptr, y, s);
}

}  // namespace lc
