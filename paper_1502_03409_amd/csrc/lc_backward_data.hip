// lc_backward_data: dx[b,p] = sum over fields l containing pixel p, sum_f w[l,k(p,l),f] * dy[b,l,f]
// (Eq. 1's reconstruction "W^T h": the overlap-add of every field's back-projection).
//
// Gather form, no atomics.  The image is cut into S x S x C "cells" (cell (ri,wi) = rows ri*S..ri*S+S-1,
// columns wi*S..wi*S+S-1).  All pixels of a cell are covered by the same fields (ri-a, wi-a'),
// a, a' < ceil(R/S), and inside field (ri-a, wi-a') the cell is the patch block kh = S*a+dr,
// kw = S*a'+dw.  So one cell is a dense contraction
//     dx_cell[b][n=(dr,dw,c)] = sum_{a,a',f} dy[b][(ri-a,wi-a')][f] * w[(ri-a,wi-a')][k(a,a',n)][f]
// of length ceil(R/S)^2 * F, in which every weight is used exactly once.
//
// A workgroup (4 waves) owns NCELL horizontally adjacent cells x 4/NCELL blocks of 16*NT cell values
// and a batch tile of 16*MT images.  dy of the covering fields of one field row is staged in LDS and
// shared by the waves (adjacent cells share most of their fields).  Weights go straight from global
// memory into the MFMA B operand: lane (n,kk) reads VF consecutive f of row k(n), and the A operand
// reads the matching f of dy from LDS, so the contraction index of the MFMA is a permutation of f.
#include <algorithm>

#include "lc_common.hpp"

namespace lc {

// T: storage type of dy and w (float, or bf16 bit patterns widened on their way in).
template <int MT, int NT, int NCELL, int VF, typename T>
__global__ __launch_bounds__(256) void lc_bwd_data_kernel(Geom g, const T *__restrict__ dy,
                                                          const T *__restrict__ w, float *__restrict__ dx,
                                                          int strips_per_row, int AP, int JW, int fcs, int rs) {
    typedef typename RawVec<T, 4>::V WV4;     // four consecutive filters of one weight row as loaded
    constexpr int BT = 16 * MT, NNW = 4 / NCELL;
    extern __shared__ __attribute__((aligned(16))) float dys[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, kk = lane >> 4;
    const int FC = 1 << fcs, SC = g.S * g.C, NCV = g.S * SC;
    const int work = remap_xcd(blockIdx.x, gridDim.x);
    const int ri = work / strips_per_row, wi0 = (work - ri * strips_per_row) * NCELL;
    const int b0 = blockIdx.z * BT;
    const int wc = wave % NCELL, wn = wave / NCELL;
    const int wi = wi0 + wc;
    const int CW = (g.W + g.S - 1) / g.S;
    const int n0 = (blockIdx.y * NNW + wn) * NT * 16;
    const bool active = (wi < CW) && (n0 < NCV);

    // per-lane decomposition of the cell values this lane supplies weights for
    int dr[NT], dwv[NT], kn[NT];
    bool nok[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int n = n0 + nt * 16 + m;
        nok[nt] = active && n < NCV;
        const int nc = nok[nt] ? n : 0;
        dr[nt] = nc / SC;
        const int rem = nc - dr[nt] * SC;
        dwv[nt] = rem / g.C;
        kn[nt] = dr[nt] * g.RC + rem;
    }

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int rowlen = JW * FC;                            // staged floats per image
    const int q_first = tid % rowlen, b_first = tid / rowlen, dq = 256 % rowlen, db = 256 / rowlen;
    // staged window of JW = min(NCELL + AP - 1, LW) field columns: it starts at the strip's first covering
    // field, moved into the grid (a layer with few fields per row stages no columns that do not exist)
    const int jlo = min(max(wi0 - (AP - 1), 0), g.LW - JW);
    const size_t dyimg = (size_t)g.L * g.F;

    for (int a = 0; a < AP; ++a) {
        const int i = ri - a;
        if (i < 0 || i >= g.LH) continue;                  // uniform over the workgroup
        for (int fc0 = 0; fc0 < g.F; fc0 += FC) {
            __syncthreads();
            {
                int q = q_first, bb = b_first;
                while (bb < BT) {
                    const int js = q >> fcs, f = fc0 + (q & (FC - 1)), j = jlo + js;
                    float v = 0.f;
                    if (j >= 0 && j < g.LW && f < g.F && b0 + bb < g.B)
                        v = ld_f32(dy + (size_t)(b0 + bb) * dyimg + (size_t)(i * g.LW + j) * g.F + f);
                    dys[bb * rs + q] = v;
                    q += dq;
                    bb += db;
                    if (q >= rowlen) { q -= rowlen; ++bb; }
                }
            }
            __syncthreads();
            if (!active) continue;
            for (int ap = 0; ap < AP; ++ap) {
                const int j = wi - ap;
                if (j < 0 || j >= g.LW) continue;          // uniform over the wave
                const int js = j - jlo;
                const T *wl = w + ((size_t)(i * g.LW + j) * g.K + (size_t)g.S * a * g.RC + g.S * ap * g.C) * g.F + fc0;
                bool ok[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    ok[nt] = nok[nt] && (g.S * a + dr[nt] < g.R) && (g.S * ap + dwv[nt] < g.R);
                const float *arow = dys + m * rs + js * FC + VF * kk;
                for (int fq = 0; fq < FC; fq += 4 * VF) {
                    if (fc0 + fq >= g.F) break;
                    float av[MT][VF], bv[NT][VF];
                    const int fl = fq + VF * kk;           // this lane's first f inside the chunk
                    if (VF == 4) {
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) {
                            f32x4 t = (f32x4){0.f, 0.f, 0.f, 0.f};
                            if (ok[nt] && fc0 + fl < g.F) t = raw_widen4<T>(*(const WV4 *)(wl + (size_t)kn[nt] * g.F + fl));
                            bv[nt][0] = t[0]; bv[nt][1 % VF] = t[1]; bv[nt][2 % VF] = t[2]; bv[nt][3 % VF] = t[3];
                        }
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            const float4 t = *(const float4 *)(arow + mt * 16 * rs + fq);
                            av[mt][0] = t.x; av[mt][1 % VF] = t.y; av[mt][2 % VF] = t.z; av[mt][3 % VF] = t.w;
                        }
                    } else {
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            bv[nt][0] = (ok[nt] && fc0 + fl < g.F) ? ld_f32(wl + (size_t)kn[nt] * g.F + fl) : 0.f;
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) av[mt][0] = arow[mt * 16 * rs + fq];
                    }
#pragma unroll
                    for (int t = 0; t < VF; ++t)
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                            for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = mfma16(av[mt][t], bv[nt][t], acc[mt][nt]);
                }
            }
        }
    }

    if (!active) return;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        if (!nok[nt]) continue;
        const int row = ri * g.S + dr[nt], col = wi * g.S + dwv[nt];
        if (row >= g.H || col >= g.W) continue;
        const int rem = kn[nt] - dr[nt] * g.RC;            // dw*C + c
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


// ---------------------------------------------------------------------------------------------
// Fast path (F % 16 == 0, R % S == 0).  Same cell-gather decomposition with the pipeline of the forward
// kernel: a chunk is one field row (a) and 16 filters (fh) of every field the strip of cells touches;
// the next chunk's dy travels through registers into the second LDS buffer while the current one is
// multiplied (one barrier per chunk); the weights of a whole chunk are in flight ahead of their use.
// Per step a' a wave multiplies dy[16*MT images][16 f] of field (ri-a, wi-a') with the S x S x C block of that field's filters:
// lane (n,kk) loads w[k(n)][fh*16 + 4kk .. +3] as one dwordx4, and lane (m,kk) reads the same four f
// of image m from LDS, so component t of both vectors is contraction index 4kk+t of MFMA number t.
// Fields outside the grid are staged as zeros (their weights are read from a clamped, valid address),
// so the inner loop has no divergent branches.
//
// The loop is written so that it holds next to no vector ALU instructions.  A SIMD issues matrix and vector ALU
// instructions through one port, and a wave whose next MFMA waits for the matrix pipe holds that port: address
// arithmetic of the other wave on the SIMD does not slip in between, it runs when the MFMAs are through and
// its time adds to theirs (measured with cycle stamps: a step of 16 MFMAs per wave took 640 cycles where 512
// were matrix work, and the staging between chunks another 2000).  Hence
//   - the wave index is read into a scalar register, so the weight pointers (the same for every lane up to the
//     lane's own offset kn) are scalar arithmetic and the loads take a scalar base plus a 32-bit lane offset;
//   - where a lane's staging slots lie, in global memory relative to the chunk and in LDS, does not depend
//     on the chunk: both offsets are worked out once; a slot that stages nothing (a field column outside the grid,
//     an image past the batch) loads from the chunk's first vector and writes to a dump vector of the lane's own
//     behind the buffer, and its place in the buffer is zeroed once, before the loop;
//   - the LDS reads of a step differ from those of the next by a compile-time offset.
template <int MT, int NT, int NCELL, int AP, int NW = 4, typename T = float>
__global__ __launch_bounds__(64 * NW, NW == 8 ? 2 : 1) void lc_bwd_data_fast_kernel(
    Geom g, const T *__restrict__ dy, const T *__restrict__ w, float *__restrict__ dx, int strips_per_row,
    int RS, int nbt) {
    typedef typename RawVec<T, 4>::V XV;      // four consecutive dy or w values as loaded (fp32, or bf16 bit patterns)
    typedef const __attribute__((address_space(1))) XV *g4_ptr;
    typedef const __attribute__((address_space(1))) T *gf_ptr;
    typedef const __attribute__((address_space(1))) char *gb_ptr;
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    constexpr int BT = 16 * MT, JW = NCELL + AP - 1, R4 = JW * 4;   // R4: 4-element vectors per image and chunk
    constexpr int NTHR = 64 * NW;                                   // NW waves: NCELL cells x NW/NCELL value blocks
    constexpr int NSLOT = (BT * R4 + NTHR - 1) / NTHR;
    constexpr int ES = sizeof(T);
    extern __shared__ __attribute__((aligned(16))) float dys_f32[];
    T *dys = (T *)dys_f32;                    // staged dy in the operands' own storage type; RS counts elements
    constexpr bool kHalf = sizeof(T) == 2;    // bf16: one 16x16x16 bf16 MFMA takes the place of four fp32 steps
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 15, kk = lane >> 4;
    const int SC = g.S * g.C, NCV = g.S * SC;
    // Work order.  Cell rows that all AP field rows cover cost the same and come first: each XCD walks a
    // contiguous range of them, and the batch tiles of one strip are neighbours in that order, so the second
    // one finds the strip's weights in that XCD's L2.  The rows at the top and bottom edge, covered by fewer
    // field rows and cheaper in proportion, come last in plain hardware order, which deals them out evenly:
    // in one contiguous walk the XCDs holding the edge rows would run dry while the others still work.
    const int r_lo = AP - 1, n_in = g.LH > r_lo ? g.LH - r_lo : 0;   // interior cell rows [r_lo, LH)
    const int per_row = strips_per_row * nbt, n_first = n_in * per_row;
    int ri, t_id;
    if ((int)blockIdx.x < n_first) {
        t_id = remap_xcd(blockIdx.x, n_first);
        ri = r_lo + t_id / per_row;
    } else if (n_in > 0) {
        t_id = blockIdx.x - n_first;
        const int rb = t_id / per_row;
        ri = rb < r_lo ? rb : g.LH + (rb - r_lo);
    } else {
        t_id = remap_xcd(blockIdx.x, gridDim.x);
        ri = t_id / per_row;
    }
    const int wi0 = ((t_id / nbt) % strips_per_row) * NCELL;
    const int b0 = (t_id % nbt) * BT;
    const int wc = wave % NCELL;
    const int wi = wi0 + wc;
    const int n0 = (blockIdx.y * (NW / NCELL) + wave / NCELL) * NT * 16;
    const int nfh = g.F >> 4;

    // cell values this lane supplies weights for / stores
    unsigned kn[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int nn = n0 + nt * 16 + m;
        const int nc = nn < NCV ? nn : 0;
        const int dr = nc / SC;
        kn[nt] = (unsigned)((dr * g.RC + (nc - dr * SC)) * g.F + 4 * kk) * ES;    // byte offset inside a field's K x F matrix
    }

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // chunks: (a, fh) with a valid field row i = ri - a
    const int a_lo = max(0, ri - (g.LH - 1)), a_hi = min(AP - 1, ri);   // inclusive; empty if a_lo > a_hi
    const int nchunks = a_hi >= a_lo ? (a_hi - a_lo + 1) * nfh : 0;
    const int jlo = wi0 - (AP - 1);
    const size_t dyimg = (size_t)g.L * g.F;

    // LDS: two halves, each a buffer of BT rows of RS elements followed by one dump vector per lane
    const int HALF = BT * RS + NTHR * 4;
    constexpr int DV = NTHR % R4, DB = NTHR / R4;
    unsigned goff[NSLOT], loff[NSLOT];   // byte offsets of a slot: from the chunk's first vector / inside a half
    {
        int v = tid % R4, b = tid / R4;
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            const int j = jlo + (v >> 2);
            const bool ok = b < BT && b0 + b < g.B && j >= 0 && j < g.LW;
            goff[q] = ok ? (unsigned)(((size_t)b * dyimg + (size_t)j * g.F + (v & 3) * 4) * ES) : 0u;
            loff[q] = (ok ? (unsigned)(b * RS + v * 4) : (unsigned)(BT * RS + tid * 4)) * ES;
            if (b < BT && !ok) {
                *(XV *)(dys + b * RS + v * 4) = XV{};
                *(XV *)(dys + HALF + b * RS + v * 4) = XV{};
            }
            v += DV; b += DB;
            if (v >= R4) { v -= R4; ++b; }
        }
    }
    XV st[NSLOT];
    // the chunk's first vector: image b0, field row ri - a, field column 0, filters fh*16..
    auto chunk_base = [&](int a, int fh) -> gf_ptr {
        return (gf_ptr)dy + (size_t)b0 * dyimg + (size_t)((ri - a) * g.LW) * g.F + fh * 16;
    };
    auto stage_load = [&](gf_ptr base) {
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) st[q] = *(g4_ptr)((gb_ptr)base + goff[q]);
    };
    auto stage_store = [&](int buf) {
        T *half = dys + buf * HALF;
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            // two 8-byte stores: 16-byte LDS stores of a row-major tile run into bank conflicts
            T *dst = (T *)((char *)half + loff[q]);
            if constexpr (kHalf) {
                *(XV *)dst = st[q];
            } else {
                *(f32x2 *)dst = (f32x2){st[q][0], st[q][1]};
                *(f32x2 *)(dst + 2) = (f32x2){st[q][2], st[q][3]};
            }
        }
    };
    // weights of step a' of chunk (a, fh): field (ri-a, wi-a') clamped into the grid; the same for every lane
    auto wbase = [&](int a, int fh, int ap) -> gf_ptr {
        int j = wi - ap;
        j = j < 0 ? 0 : (j >= g.LW ? g.LW - 1 : j);
        return (gf_ptr)w + ((size_t)((ri - a) * g.LW + j) * g.K + (size_t)g.S * a * g.RC + g.S * ap * g.C) * g.F +
               fh * 16;
    };
    // chunk c is (a, fh) = (a_lo + c / nfh, c % nfh), counted along rather than divided out
    struct Chunk { int a, fh; };
    auto after = [&](Chunk c) -> Chunk { return c.fh + 1 == nfh ? Chunk{c.a + 1, 0} : Chunk{c.a, c.fh + 1}; };

    if (nchunks > 0) {
        // weight ring: slot a' holds the weights of step a' of the current chunk and is refilled, right
        // after its use, with step a' of the next chunk: loads run one whole chunk ahead of the MFMAs
        XV wb[AP][NT];
#pragma unroll
        for (int ap = 0; ap < AP; ++ap) {
            gf_ptr p0 = wbase(a_lo, 0, ap);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) wb[ap][nt] = *(g4_ptr)((gb_ptr)p0 + kn[nt]);
        }
        // two LDS buffers: chunk c is read from buffer c & 1 while chunk c+1, whose loads were issued a whole
        // chunk earlier, goes from the staging registers into the other one; one barrier per chunk
        Chunk c0 = {a_lo, 0}, c1 = after(c0), c2 = after(c1);     // chunks c, c+1, c+2
        stage_load(chunk_base(c0.a, c0.fh));
        stage_store(0);
        if (nchunks > 1) stage_load(chunk_base(c1.a, c1.fh));
        __syncthreads();
        // the lane's dy vector of image m + 16 mt under the wave's cell at step a' lies at
        // abase + mt*16*RS + (AP-1-a')*16: field column wc - a' + AP - 1 of the staged strip
        const T *abase = dys + m * RS + 4 * kk + wc * 16;
        for (int c = 0; c < nchunks; ++c) {
            const T *arow = abase + (c & 1) * HALF;
            const bool more = c + 1 < nchunks;
            const Chunk cw = more ? c1 : c0;      // the last chunk reloads its own weights: a valid address, the values are not used
            // The A operands of step a'+1 are read from LDS before the MFMAs of step a': left to itself the compiler
            // issues every LDS read right in front of the MFMAs that use it and waits for it there.
            XV av[2][MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) av[0][mt] = *(const XV *)(arow + mt * 16 * RS + (AP - 1) * 16);
#pragma unroll
            for (int ap = 0; ap < AP; ++ap) {
                if (ap + 1 < AP) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        av[(ap + 1) & 1][mt] = *(const XV *)(arow + mt * 16 * RS + (AP - 2 - ap) * 16);
                }
                __builtin_amdgcn_sched_barrier(0);
                // a field column outside the grid contributes nothing: skip its MFMAs (the same for the whole wave)
                if (wi - ap >= 0 && wi - ap < g.LW) {
                    if constexpr (kHalf) {
                        // the vectors already are the operands: four consecutive f of image m / of cell value n
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                            for (int nt = 0; nt < NT; ++nt)
                                acc[mt][nt] = mfma16_bf16(av[ap & 1][mt], wb[ap][nt], acc[mt][nt]);
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t)
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                                for (int nt = 0; nt < NT; ++nt)
                                    acc[mt][nt] = mfma16(av[ap & 1][mt][t], wb[ap][nt][t], acc[mt][nt]);
                    }
                }
                gf_ptr pn = wbase(cw.a, cw.fh, ap);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) wb[ap][nt] = *(g4_ptr)((gb_ptr)pn + kn[nt]);
                __builtin_amdgcn_sched_barrier(0);
            }
            // the other buffer was last read in chunk c-1, which every wave left at the previous barrier
            if (more) stage_store((c + 1) & 1);
            if (c + 2 < nchunks) stage_load(chunk_base(c2.a, c2.fh));
            c0 = c1; c1 = c2; c2 = after(c2);
            __syncthreads();
        }
    }

    if (wi * g.S >= g.W) return;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
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

// ---------------------------------------------------------------------------------------------
// The pipelined kernel for fp32 operands with a hand-kept memory schedule.  Same decomposition, chunks and steps as
// lc_bwd_data_fast_kernel; what differs is how the operands travel:
//   - dy goes from global memory straight into LDS (16 bytes per lane, lane i of a wave's load lands 16 i bytes past
//     the load's LDS base): no staging registers, no LDS stores, no address arithmetic per chunk.  An LDS buffer is the
//     batch tile's rows one after the other, each row JW field columns x 16 filters plus one pad vector (row stride
//     16 bytes past a multiple of 64: the 16 rows a wave reads at once start four banks apart), so vector P of the
//     buffer belongs to lane P % NTHR of load P / NTHR, and where that lane reads from does not depend on the chunk.
//     A lane whose vector stages nothing (a field column outside the grid, an image past the batch) is switched off
//     for the load and its vector is zeroed once, before the loop; lanes on pad vectors and past the last row load
//     the chunk's first vector into space nobody reads, so every wave's every load has a live lane and the number
//     of loads in flight is the same for all waves;
//   - the loads are inline assembly, which the compiler's wait insertion does not see, and every wait on them is
//     written out below.  The memory counter counts loads in program order, and the order is fixed:
//         chunk c:  [NSLOT dy loads of chunk c+1]  then per step a': wait, MFMAs, [NT weight loads of step a', chunk c+1]
//     so at step a' the weights of (c, a') are followed by AP*NT - NT + NSLOT younger loads (those may stay in flight),
//     and at the chunk's end the dy loads are followed by AP*NT: each wait is for a load issued a whole chunk
//     earlier.  The compiler, not knowing the order of chunks, waits for all but the seven youngest loads at every step,
//     which at the first steps of a chunk are the dy loads just issued.
// The last chunk loads its own dy and weights once more (valid addresses; the values are not used) so that the
// counts hold in every iteration.
template <int MT, int NT, int NCELL, int AP, int NW, int NBUF>
__global__ __launch_bounds__(64 * NW, (NW == 8 ? 2 : 1) * (3 - NBUF)) void lc_bwd_data_direct_kernel(
    Geom g, const float *__restrict__ dy, const float *__restrict__ w, float *__restrict__ dx, int strips_per_row,
    int nbt) {
    constexpr int BT = 16 * MT, JW = NCELL + AP - 1, R4 = JW * 4;   // R4: 4-filter vectors per image and chunk
    constexpr int RV = R4 + 1, RS = RV * 4;                          // LDS row: R4 vectors and a pad; RS floats
    constexpr int NTHR = 64 * NW;                                   // NW waves: NCELL cells x NW/NCELL value blocks
    constexpr int NV = BT * RV, NSLOT = (NV + NTHR - 1) / NTHR;     // vectors per buffer, loads per lane and chunk
    constexpr int BUF = NSLOT * NTHR * 4;                           // floats per buffer, the last load's slack included
    static_assert(RV <= 64, "every wave's load must cover a pad vector");
    static_assert(AP * NT - NT + NSLOT <= 63 && AP * NT <= 63, "the memory counter has six bits");
    extern __shared__ __attribute__((aligned(16))) float dys[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 15, kk = lane >> 4;
    const int SC = g.S * g.C, NCV = g.S * SC;
    // work order as in lc_bwd_data_fast_kernel: full-cost cell rows first, a contiguous range per XCD with the batch
    // tiles of a strip next to each other; the cheaper rows at the top and bottom edge last, dealt out evenly
    const int r_lo = AP - 1, n_in = g.LH > r_lo ? g.LH - r_lo : 0;
    const int per_row = strips_per_row * nbt, n_first = n_in * per_row;
    int ri, t_id;
    if ((int)blockIdx.x < n_first) {
        t_id = remap_xcd(blockIdx.x, n_first);
        ri = r_lo + t_id / per_row;
    } else if (n_in > 0) {
        t_id = blockIdx.x - n_first;
        const int rb = t_id / per_row;
        ri = rb < r_lo ? rb : g.LH + (rb - r_lo);
    } else {
        t_id = remap_xcd(blockIdx.x, gridDim.x);
        ri = t_id / per_row;
    }
    const int wi0 = ((t_id / nbt) % strips_per_row) * NCELL;
    const int b0 = (t_id % nbt) * BT;
    const int wc = wave % NCELL;
    const int wi = wi0 + wc;
    const int n0 = (blockIdx.y * (NW / NCELL) + wave / NCELL) * NT * 16;
    const int nfh = g.F >> 4;

    // cell values this lane supplies weights for / stores
    unsigned kn[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int nn = n0 + nt * 16 + m;
        const int nc = nn < NCV ? nn : 0;
        const int dr = nc / SC;
        kn[nt] = (unsigned)((dr * g.RC + (nc - dr * SC)) * g.F + 4 * kk) * 4u;    // byte offset inside a field's K x F matrix
    }

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // chunks: (a, fh) with a valid field row i = ri - a
    const int a_lo = max(0, ri - (g.LH - 1)), a_hi = min(AP - 1, ri);   // inclusive; empty if a_lo > a_hi
    const int nchunks = a_hi >= a_lo ? (a_hi - a_lo + 1) * nfh : 0;
    const int jlo = wi0 - (AP - 1);
    const size_t dyimg = (size_t)g.L * g.F;

    if (nchunks > 0) {
        // weights of step a' of chunk (a, fh): field (ri-a, wi-a') clamped into the grid; the same for every lane.
        // Row (ri-a) of the grid, kernel row S*a and filters fh*16.. give the chunk's pointer; the step adds the field
        // column and kernel column, which no chunk changes: wstep[a'] is worked out once.
        size_t wstep[AP];
#pragma unroll
        for (int ap = 0; ap < AP; ++ap) {
            int j = wi - ap;
            j = j < 0 ? 0 : (j >= g.LW ? g.LW - 1 : j);
            wstep[ap] = ((size_t)j * g.K + (size_t)(g.S * ap * g.C)) * g.F * 4;
        }
        auto wchunk = [&](int a, int fh) -> gbyte_ptr {
            return (gbyte_ptr)(w + ((size_t)((ri - a) * g.LW) * g.K + (size_t)g.S * a * g.RC) * g.F + fh * 16);
        };
        // weight ring: slot a' holds the weights of step a' of the current chunk and is refilled, right
        // after its use, with step a' of the next chunk: loads run one whole chunk ahead of the MFMAs
        f32x4 wb[AP][NT];
#pragma unroll
        for (int ap = 0; ap < AP; ++ap) {
            gbyte_ptr p0 = wchunk(a_lo, 0) + wstep[ap];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) wb[ap][nt] = load_nowait<4>(p0, kn[nt]);
        }

        // where this lane's vector of load q comes from (bytes past the chunk's first vector), whether it loads at
        // all; vectors that stage nothing are zeroed in both buffers
        unsigned goff[NSLOT];
        bool live[NSLOT];
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            const int P = q * NTHR + tid, b = P / RV, v = P - b * RV;
            const int j = jlo + (v >> 2);
            const bool data = P < NV && v < R4;
            const bool ok = data && b0 + b < g.B && j >= 0 && j < g.LW;
            goff[q] = ok ? (unsigned)(((size_t)b * dyimg + (size_t)j * g.F + (v & 3) * 4) * 4) : 0u;
            live[q] = ok || !data;
            if (data && !ok) {
                *(f32x4 *)(dys + P * 4) = (f32x4){0.f, 0.f, 0.f, 0.f};
                if constexpr (NBUF == 2) *(f32x4 *)(dys + BUF + P * 4) = (f32x4){0.f, 0.f, 0.f, 0.f};
            }
        }
        const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) float *)dys + wave * 64 * 16;
        // chunk c is (a, fh) = (a_lo + c / nfh, c % nfh), counted along rather than divided out
        struct Chunk { int a, fh; };
        auto after = [&](Chunk c) -> Chunk { return c.fh + 1 == nfh ? Chunk{c.a + 1, 0} : Chunk{c.a, c.fh + 1}; };
        auto stage = [&](Chunk ch, int buf) {
            gbyte_ptr base = (gbyte_ptr)(dy + (size_t)b0 * dyimg + (size_t)((ri - ch.a) * g.LW) * g.F + ch.fh * 16);
            const unsigned l = lds0 + buf * (BUF * 4);
#pragma unroll
            for (int q = 0; q < NSLOT; ++q)
                if (live[q]) load_lds16(base, goff[q], l + q * (NTHR * 16));
        };

        // With two buffers, the dy loads of the next chunk go out a few at a time (SPS per step) behind the MFMAs of the
        // first half of the steps instead of all at the chunk's start, where they queue up in the compute unit's one
        // address unit with the waves, which issue in order, standing behind them; in the first half, so that the last
        // one has half a chunk to land.
        constexpr bool kSpread = NBUF == 2;
        constexpr int NSP = AP / 2 > 0 ? AP / 2 : 1, SPS = (NSLOT + NSP - 1) / NSP;
        constexpr int kLastDmaStep = (NSLOT - 1) / SPS;
        auto dma_in_step = [&](int ap) -> int {
            const int lo = ap * SPS, hi = (ap + 1) * SPS < NSLOT ? (ap + 1) * SPS : NSLOT;
            return hi > lo ? hi - lo : 0;
        };
        Chunk c0 = {a_lo, 0}, c1 = after(c0);     // chunks c and c+1
        // the lane's dy vector of image m + 16 mt under the wave's cell at step a' lies at
        // abase + mt*16*RS + (AP-1-a')*16: field column wc - a' + AP - 1 of the staged strip
        const float *abase = dys + m * RS + 4 * kk + wc * 16;
        if constexpr (NBUF == 2) {
            stage(c0, 0);
            wait_loads<0>();
            __syncthreads();
        }
        for (int c = 0; c < nchunks; ++c) {
            const Chunk cn = c + 1 < nchunks ? c1 : c0;
            const float *arow = abase;
            gbyte_ptr dnext = (gbyte_ptr)(dy + (size_t)b0 * dyimg + (size_t)((ri - cn.a) * g.LW) * g.F + cn.fh * 16);
            const unsigned lnext = lds0 + ((c + 1) & 1) * (BUF * 4);
            if constexpr (NBUF == 2) {
                if constexpr (!kSpread) stage(cn, (c + 1) & 1);
                arow += (c & 1) * BUF;
            } else {
                // one buffer, and several workgroups on a compute unit to work while this one waits for its dy
                if (c > 0) __syncthreads();      // everybody is through with chunk c-1
                stage(c0, 0);
                wait_loads<0>();                 // with it, the weights of this chunk have landed
                __syncthreads();
            }
            f32x4 av[2][MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) av[0][mt] = *(const f32x4 *)(arow + mt * 16 * RS + (AP - 1) * 16);
            gbyte_ptr wn = wchunk(cn.a, cn.fh);
#pragma unroll
            for (int ap = 0; ap < AP; ++ap) {
                const bool inside = wi - ap >= 0 && wi - ap < g.LW;   // a field column outside the grid contributes
                                                                      // nothing: its MFMAs are skipped (by the whole wave)
                if constexpr (NBUF == 2) {
                    // behind the weights of step a': those of the other AP-1 steps and every dy load but this step's own
                    // (the loop is unrolled: a' is a constant by the time this is compiled)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        wait_loads_minus<AP * NT - NT + NSLOT, SPS>(kSpread ? dma_in_step(ap) : 0, wb[ap][nt]);
                }
                __builtin_amdgcn_sched_barrier(0);
                auto mfmas = [&](int t) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            acc[mt][nt] = mfma16(av[ap & 1][mt][t], wb[ap][nt][t], acc[mt][nt]);
                };
                if (inside) { mfmas(0); mfmas(1); }
                __builtin_amdgcn_sched_barrier(0);
                // Issued behind the first MFMAs, the LDS reads of the next step and the pointer arithmetic of the
                // weight loads run while the matrix pipe works them off: a wave issues in order, and whatever stands
                // in front of the step's first MFMA is time the pipe idles when the SIMD's other wave is not ready.
                if (ap + 1 < AP) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        av[(ap + 1) & 1][mt] = *(const f32x4 *)(arow + mt * 16 * RS + (AP - 2 - ap) * 16);
                }
                gbyte_ptr pn = wn + wstep[ap];
                __builtin_amdgcn_sched_barrier(0);
                if (inside) { mfmas(2); mfmas(3); }
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (kSpread) {
#pragma unroll
                    for (int q = ap * SPS; q < (ap + 1) * SPS && q < NSLOT; ++q)
                        if (live[q]) load_lds16(dnext, goff[q], lnext + q * (NTHR * 16));
                }
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) wb[ap][nt] = load_nowait<4>(pn, kn[nt]);
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (NBUF == 2) {
                // this lane's dy loads of the next chunk have landed (the AP*NT weight loads behind them may fly on);
                // behind the barrier, everybody's have, and everybody is through with the buffer the chunk after next
                // overwrites
                if constexpr (kSpread) wait_loads<(AP - kLastDmaStep) * NT>();
                else wait_loads<AP * NT>();
                __syncthreads();
            }
            c0 = c1; c1 = after(c1);
        }
        // the weights loaded last are not used: they must have landed before their registers are given up
#pragma unroll
        for (int ap = 0; ap < AP; ++ap)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) wait_loads<0>(wb[ap][nt]);
    }

    if (wi * g.S >= g.W) return;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
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

// ---------------------------------------------------------------------------------------------
// Layers whose filters come in blocks of 32 (32 filters of a row of w[l], or of a field's dy, are one 128-byte
// line).  The pipelined kernel above reads such a line in two halves a whole chunk apart, and the memory side moves
// whole lines: by the time the second half is asked for, the line has left the L2 again and is fetched a second
// time.  Here a chunk is one field row with 32 filters, so both halves of a line are read within one step of each
// other: the staged dy arrives as whole lines, and the weight ring (RING half-steps deep) asks for the halves of a
// row in consecutive half-steps.  The chunk is twice as large, so there is one LDS buffer and two barriers per
// chunk: the next chunk waits in the staging registers while the current one is multiplied.  With those 64
// staging registers a ring of five half-steps no longer fits 256 registers (5 values spilled and reloaded inside
// the loop, each reload waiting for every load issued before it); two half-steps fit and measured faster
// (5 x 5 covering fields of 32 filters, 104 x 104 x 12 input, batch 128: 233 -> 225 us; one half-step: 264 us).
template <int MT, int NT, int NCELL, int AP, int RING>
__global__ __launch_bounds__(256, 2) void lc_bwd_data_line_kernel(Geom g, const float *__restrict__ dy,
                                                                  const float *__restrict__ w,
                                                                  float *__restrict__ dx, int strips_per_row,
                                                                  int RS, int nbt) {
    typedef const __attribute__((address_space(1))) f32x4 *g4_ptr;
    typedef const __attribute__((address_space(1))) float *gf_ptr;
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    constexpr int BT = 16 * MT, JW = NCELL + AP - 1, R4 = JW * 8;   // R4: float4 per image and chunk (32 f per field)
    constexpr int NTHR = 256, NSLOT = (BT * R4 + NTHR - 1) / NTHR, NHS = 2 * AP;
    static_assert(NHS % RING == 0, "the ring's slot pattern must repeat every chunk");
    extern __shared__ __attribute__((aligned(16))) float dys_line[];
    float *dys = dys_line;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, kk = lane >> 4;
    const int SC = g.S * g.C, NCV = g.S * SC;
    // work order as in the pipelined kernel: full-cost cell rows first, a contiguous range per XCD with the batch
    // tiles of a strip next to each other; the cheaper rows at the top and bottom edge last, dealt out evenly
    const int r_lo = AP - 1, n_in = g.LH > r_lo ? g.LH - r_lo : 0;
    const int per_row = strips_per_row * nbt, n_first = n_in * per_row;
    int ri, t_id;
    if ((int)blockIdx.x < n_first) {
        t_id = remap_xcd(blockIdx.x, n_first);
        ri = r_lo + t_id / per_row;
    } else if (n_in > 0) {
        t_id = blockIdx.x - n_first;
        const int rb = t_id / per_row;
        ri = rb < r_lo ? rb : g.LH + (rb - r_lo);
    } else {
        t_id = remap_xcd(blockIdx.x, gridDim.x);
        ri = t_id / per_row;
    }
    const int wi0 = ((t_id / nbt) % strips_per_row) * NCELL;
    const int b0 = (t_id % nbt) * BT;
    const int wc = wave % NCELL;
    const int wi = wi0 + wc;
    const int n0 = (blockIdx.y * (4 / NCELL) + wave / NCELL) * NT * 16;

    int kn[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int nn = n0 + nt * 16 + m;
        const int nc = nn < NCV ? nn : 0;
        const int dr = nc / SC;
        kn[nt] = (dr * g.RC + (nc - dr * SC)) * g.F + 4 * kk;
    }

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // chunks: (a, fp) = the valid field rows i = ri - a, 32 filters fp*32 .. fp*32+31 at a time
    const int a_lo = max(0, ri - (g.LH - 1)), a_hi = min(AP - 1, ri);
    const int nfp = g.F >> 5;
    const int nchunks = a_hi >= a_lo ? (a_hi - a_lo + 1) * nfp : 0;
    const int jlo = wi0 - (AP - 1);
    const size_t dyimg = (size_t)g.L * g.F;

    const int v0 = tid % R4, bq0 = tid / R4;
    constexpr int DV = NTHR % R4, DB = NTHR / R4;
    f32x4 st[NSLOT];
    auto stage_load = [&](int c) {
        const int ca = c / nfp, fp = c - ca * nfp;
        const float *base = dy + (size_t)b0 * dyimg + (size_t)((ri - (a_lo + ca)) * g.LW) * g.F + fp * 32;
        int v = v0, b = bq0;
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            const int j = jlo + (v >> 3);
            f32x4 t = (f32x4){0.f, 0.f, 0.f, 0.f};
            if (b < BT && b0 + b < g.B && j >= 0 && j < g.LW)
                t = *(g4_ptr)(base + (size_t)b * dyimg + j * g.F + (v & 7) * 4);
            st[q] = t;
            v += DV; b += DB;
            if (v >= R4) { v -= R4; ++b; }
        }
    };
    auto stage_store = [&]() {
        int v = v0, b = bq0;
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            if (b < BT) {
                float *dst = dys + b * RS + v * 4;      // 8-byte stores: 16-byte ones of a row-major tile conflict
                *(f32x2 *)dst = (f32x2){st[q][0], st[q][1]};
                *(f32x2 *)(dst + 2) = (f32x2){st[q][2], st[q][3]};
            }
            v += DV; b += DB;
            if (v >= R4) { v -= R4; ++b; }
        }
    };
    // weights of half-step hs = 2 a' + fh of chunk c: filters 16 fh .. 16 fh + 15 of field (ri-a, wi-a'), clamped
    auto wbase = [&](int c, int hs) -> gf_ptr {
        const int ca = c / nfp, fp = c - ca * nfp;
        const int a = a_lo + ca, ap = hs >> 1;
        int j = wi - ap;
        j = j < 0 ? 0 : (j >= g.LW ? g.LW - 1 : j);
        return (gf_ptr)w + ((size_t)((ri - a) * g.LW + j) * g.K + (size_t)g.S * a * g.RC + g.S * ap * g.C) * g.F +
               fp * 32 + (hs & 1) * 16;
    };

    if (nchunks > 0) {
        f32x4 wb[RING][NT];
#pragma unroll
        for (int hs = 0; hs < RING; ++hs) {
            gf_ptr p0 = wbase(0, hs);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) wb[hs][nt] = *(g4_ptr)(p0 + kn[nt]);
        }
        stage_load(0);
        for (int c = 0; c < nchunks; ++c) {
            if (c > 0) __syncthreads();               // every wave has left chunk c-1
            stage_store();
            if (c + 1 < nchunks) stage_load(c + 1);
            __syncthreads();
            const float *arow = dys + m * RS + 4 * kk;
            const int cn = c + 1 < nchunks ? c + 1 : c;
#pragma unroll
            for (int hs = 0; hs < NHS; ++hs) {
                const int ap = hs >> 1, fh = hs & 1, slot = hs % RING;
                const int js = wc - ap + AP - 1;
                if (wi - ap >= 0 && wi - ap < g.LW) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const f32x4 av = *(const f32x4 *)(arow + mt * 16 * RS + js * 32 + fh * 16);
#pragma unroll
                        for (int t = 0; t < 4; ++t)
#pragma unroll
                            for (int nt = 0; nt < NT; ++nt)
                                acc[mt][nt] = mfma16(av[t], wb[slot][nt][t], acc[mt][nt]);
                    }
                }
                gf_ptr pn = hs + RING < NHS ? wbase(c, hs + RING) : wbase(cn, hs + RING - NHS);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) wb[slot][nt] = *(g4_ptr)(pn + kn[nt]);
                __builtin_amdgcn_sched_barrier(0x2 | 0x4 | 0x80);
            }
        }
    }

    if (wi * g.S >= g.W) return;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
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

namespace {

constexpr size_t kLdsTarget = 78 * 1024;

int row_stride(int rowlen, int vf) {
    // VF=4: lanes of one image row read 16 B each; stride == 4 (mod 32) spreads 8 rows over all banks.
    // VF=1: stride == 2 (mod 32), as in the forward kernel.
    const int res = vf == 4 ? 4 : 2;
    return ((rowlen + 31) / 32) * 32 + res;
}

// Host check of a lc_bwd_data_kernel launch.  tparam = {MT, NT, NCELL, VF, bytes per operand element}; arg = {strips of cells per cell row,
// AP = ceil(R/S), staged field columns JW, log2 of the filter chunk, LDS row stride}.  The kernel masks every
// ragged edge itself.
int check_backward_data_generic(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0], NT = p.tparam[1], NCELL = p.tparam[2], VF = p.tparam[3];
    const int strips = p.arg[0], AP = p.arg[1], JW = p.arg[2], fcs = p.arg[3], rs = p.arg[4];
    const int BT = 16 * MT, NNW = 4 / NCELL, NCV = g.S * g.S * g.C;
    const int CH = ceil_div(g.H, g.S), CW = ceil_div(g.W, g.S);
    LC_PLAN_REQUIRE(p, p.block == 256 && (NCELL == 1 || NCELL == 2 || NCELL == 4) && (VF == 1 || VF == 4));
    LC_PLAN_REQUIRE(p, AP == ceil_div(g.R, g.S) && JW == std::min(NCELL + AP - 1, g.LW));
    // 16-byte accesses along f need whole vectors of four filters
    LC_PLAN_REQUIRE(p, VF == 1 || g.F % 4 == 0);
    LC_PLAN_REQUIRE(p, fcs >= (VF == 4 ? 4 : 2) && fcs <= 20 && rs >= (JW << fcs) && (VF == 1 || rs % 4 == 0));
    LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)BT * rs * sizeof(float));
    LC_PLAN_REQUIRE(p, strips == ceil_div(CW, NCELL) && (long long)p.grid[0] == (long long)strips * CH);
    LC_PLAN_REQUIRE(p, (long long)p.grid[1] * NNW * NT * 16 >= NCV && (long long)(p.grid[1] - 1) * NNW * NT * 16 < NCV);
    LC_PLAN_REQUIRE(p, (long long)p.grid[2] * BT >= g.B && (long long)(p.grid[2] - 1) * BT < g.B);
    return LC_OK;
}

template <int MT, int NT, int NCELL, int VF, typename T>
int launch_one(const Geom &g, const T *dy, const T *w, float *dx, hipStream_t s) {
    constexpr int BT = 16 * MT, NNW = 4 / NCELL;
    const int AP = (g.R + g.S - 1) / g.S, JW = std::min(NCELL + AP - 1, g.LW);
    const int CH = (g.H + g.S - 1) / g.S, CW = (g.W + g.S - 1) / g.S;
    const int NCV = g.S * g.S * g.C;
    // f chunk: the largest power of two (>= 4*VF) that covers F or still fits the LDS budget
    int fcs = VF == 4 ? 4 : 2;
    while ((1 << fcs) < g.F && (size_t)BT * row_stride(JW << (fcs + 1), VF) * 4 <= kLdsTarget) ++fcs;
    const int rs = row_stride(JW << fcs, VF);
    const size_t lds = (size_t)BT * rs * sizeof(float);
    if (lds > 160 * 1024) return LC_EUNSUPPORTED;
    auto kern = lc_bwd_data_kernel<MT, NT, NCELL, VF, T>;
    const int strips = (CW + NCELL - 1) / NCELL;
    dim3 grid(strips * CH, (NCV + NNW * NT * 16 - 1) / (NNW * NT * 16), (g.B + BT - 1) / BT);
    const LaunchPlan plan = make_plan("lc_bwd_data_generic", {MT, NT, NCELL, VF, (int)sizeof(T)}, {strips, AP, JW, fcs, rs},
                                      grid, 256, lds);
    if (int rc = check_backward_data_generic(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_backward_data launch", kern, s, g, dy, w, dx, strips, AP, JW, fcs, rs);
    return LC_OK;
}

template <int MT, typename T>
int launch_mt(const Geom &g, const T *dy, const T *w, float *dx, hipStream_t s) {
    const int ntt = (g.S * g.S * g.C + 15) / 16;  // tiles of 16 cell values
    if ((g.F & 3) != 0) return launch_one<MT, 4, 1, 1>(g, dy, w, dx, s);
    if (ntt == 1) return launch_one<MT, 1, 4, 4>(g, dy, w, dx, s);
    if (ntt == 2) return launch_one<MT, 2, 4, 4>(g, dy, w, dx, s);
    if (ntt == 3) return launch_one<MT, 3, 4, 4>(g, dy, w, dx, s);
    if (ntt == 4) return launch_one<MT, 4, 4, 4>(g, dy, w, dx, s);
    if (ntt <= 8) return launch_one<MT, 4, 2, 4>(g, dy, w, dx, s);
    if (ntt % 16 > 12 || ntt % 16 == 0) return launch_one<MT, 4, 1, 4>(g, dy, w, dx, s);
    return launch_one<MT, 3, 1, 4>(g, dy, w, dx, s);
}

}  // namespace

namespace {

// Host check of a lc_bwd_data_fast_kernel or lc_bwd_data_line_kernel launch (LINE = 1: chunks of 32 filters, one LDS
// buffer; 0: chunks of 16 filters, two buffers).
// tparam = {MT, NT, NCELL, AP, NW, bytes per operand element, LINE (2: dy straight into LDS), RING, LDS buffers}; arg = {strips of cells per cell row, LDS
// row stride in elements, batch tiles}.
int check_backward_data_fast(const Geom &g, const LaunchPlan &p) {
    const int MT = p.tparam[0], NT = p.tparam[1], NCELL = p.tparam[2], AP = p.tparam[3], NW = p.tparam[4];
    const int ES = p.tparam[5], LINE = p.tparam[6];
    const int strips = p.arg[0], RS = p.arg[1], nbt = p.arg[2];
    LC_PLAN_REQUIRE(p, NCELL > 0 && NW % NCELL == 0 && (ES == 4 || ES == 2) &&
                           (LINE == 0 || (LINE == 1 && ES == 4 && NW == 4) || (LINE == 2 && ES == 4)));
    const int BT = 16 * MT, JW = NCELL + AP - 1, FCH = LINE == 1 ? 32 : 16, NCV = g.S * g.S * g.C;
    const int CH = ceil_div(g.H, g.S), CW = ceil_div(g.W, g.S);
    LC_PLAN_REQUIRE(p, (int)p.block == 64 * NW);
    // fields tile the cells exactly, AP of them across a cell; filters in whole chunks
    LC_PLAN_REQUIRE(p, g.R % g.S == 0 && AP == g.R / g.S && g.F % FCH == 0);
    // staged dy: JW field columns of FCH filters per image in one LDS row, whole vectors of four
    LC_PLAN_REQUIRE(p, RS >= JW * FCH && RS % 4 == 0);
    if (LINE == 0)        // two halves: a buffer and one dump vector per lane
        LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)2 * (BT * RS + 64 * NW * 4) * ES);
    else if (LINE == 1)   // one buffer
        LC_PLAN_REQUIRE(p, p.lds_bytes >= (size_t)BT * RS * ES);
    else {                // two buffers of whole loads (16 bytes per lane); a row is JW*4 vectors and a pad
        const int nslot = ceil_div(BT * (JW * 4 + 1), 64 * NW);
        const int NBUF = p.tparam[8];
        LC_PLAN_REQUIRE(p, (NBUF == 1 || NBUF == 2) && RS == (JW * 4 + 1) * 4 && JW * 4 + 1 <= 64 &&
                               p.lds_bytes >= (size_t)NBUF * nslot * 64 * NW * 16);
        // the kernel's waits count the loads in flight: a six-bit counter
        LC_PLAN_REQUIRE(p, AP * NT - NT + nslot <= 63 && AP * NT <= 63);
    }
    // pipelined kernels: 32-bit byte offsets of a lane's staging slots from the chunk's first vector
    LC_PLAN_REQUIRE(p, LINE == 1 || (long long)BT * g.L * g.F * ES < (1LL << 32));
    // 32-bit offsets inside a field's K x F matrix (kn) and inside one image's dy (j * F)
    LC_PLAN_REQUIRE(p, (long long)g.K * g.F < (1LL << 31) && (long long)g.LW * g.F < (1LL << 31));
    // every cell row (the rows past the last covered one get zeros), every strip of cells, every batch tile
    LC_PLAN_REQUIRE(p, strips == ceil_div(CW, NCELL) && nbt == ceil_div(g.B, BT));
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] == (long long)strips * CH * nbt);
    // the kernel's work order puts the cell rows [AP-1, LH) first and the rest behind them: all CH rows are reached
    // only if there are at least as many cell rows as that order assumes
    LC_PLAN_REQUIRE(p, CH >= g.LH + AP - 1);
    const int nblk = (NW / NCELL) * NT * 16;
    LC_PLAN_REQUIRE(p, (long long)p.grid[1] * nblk >= NCV && (long long)(p.grid[1] - 1) * nblk < NCV && p.grid[2] == 1);
    return LC_OK;
}

template <int MT, int NT, int NCELL, int AP, int RING>
int launch_line(const Geom &g, const float *dy, const float *w, float *dx, hipStream_t s) {
    constexpr int BT = 16 * MT, JW = NCELL + AP - 1;
    const int CH = (g.H + g.S - 1) / g.S, CW = (g.W + g.S - 1) / g.S;
    const int NCV = g.S * g.S * g.C;
    const int RS = JW * 32 + 4;                               // 16 bytes past a multiple of 128, as below
    const size_t lds = (size_t)BT * RS * sizeof(float);
    auto kern = lc_bwd_data_line_kernel<MT, NT, NCELL, AP, RING>;
    const int strips = (CW + NCELL - 1) / NCELL;
    const int nblk = (4 / NCELL) * NT * 16;
    const int nbt = (g.B + BT - 1) / BT;
    dim3 grid(strips * CH * nbt, (NCV + nblk - 1) / nblk);
    const LaunchPlan plan = make_plan("lc_bwd_data_line", {MT, NT, NCELL, AP, 4, 4, 1, RING}, {strips, RS, nbt}, grid, 256, lds);
    if (int rc = check_backward_data_fast(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_backward_data launch", kern, s, g, dy, w, dx, strips, RS, nbt);
    return LC_OK;
}

// fp32 operands: the kernel with dy loaded straight into LDS
template <int MT, int NT, int NCELL, int AP, int NW, int NBUF = 2>
int launch_direct(const Geom &g, const float *dy, const float *w, float *dx, hipStream_t s) {
    constexpr int BT = 16 * MT, JW = NCELL + AP - 1, RV = JW * 4 + 1, NTHR = 64 * NW;
    constexpr int NSLOT = (BT * RV + NTHR - 1) / NTHR;
    const int CH = (g.H + g.S - 1) / g.S, CW = (g.W + g.S - 1) / g.S;
    const int NCV = g.S * g.S * g.C;
    const size_t lds = (size_t)NBUF * NSLOT * NTHR * 16;
    auto kern = lc_bwd_data_direct_kernel<MT, NT, NCELL, AP, NW, NBUF>;
    const int strips = (CW + NCELL - 1) / NCELL;
    const int nblk = (NW / NCELL) * NT * 16;
    const int nbt = (g.B + BT - 1) / BT;
    dim3 grid(strips * CH * nbt, (NCV + nblk - 1) / nblk);
    const LaunchPlan plan = make_plan("lc_bwd_data_direct", {MT, NT, NCELL, AP, NW, 4, 2, AP, NBUF}, {strips, RV * 4, nbt},
                                      grid, NTHR, lds);
    if (int rc = check_backward_data_fast(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_backward_data launch", kern, s, g, dy, w, dx, strips, nbt);
    return LC_OK;
}

template <int MT, int NT, int NCELL, int AP, int NW = 4, typename T>
int launch_fast(const Geom &g, const T *dy, const T *w, float *dx, hipStream_t s) {
    if constexpr (sizeof(T) == 4) return launch_direct<MT, NT, NCELL, AP, NW>(g, dy, w, dx, s);
    constexpr int BT = 16 * MT, JW = NCELL + AP - 1;
    const int CH = (g.H + g.S - 1) / g.S, CW = (g.W + g.S - 1) / g.S;
    const int NCV = g.S * g.S * g.C;
    // row stride: 16 bytes past a multiple of 128 bytes, so that the 16 image rows a wave reads at once start
    // four banks apart (fp32: 16-byte reads of 4 f; bf16: 8-byte reads)
    const int RS = sizeof(T) == 2 ? ((JW * 16 + 63) / 64) * 64 + 8 : ((JW * 16 + 31) / 32) * 32 + 4;
    const size_t lds = (size_t)2 * (BT * RS + 64 * NW * 4) * sizeof(T);   // two halves: buffer + a dump vector per lane
    auto kern = lc_bwd_data_fast_kernel<MT, NT, NCELL, AP, NW, T>;
    const int strips = (CW + NCELL - 1) / NCELL;
    const int nblk = (NW / NCELL) * NT * 16;
    const int nbt = (g.B + BT - 1) / BT;
    dim3 grid(strips * CH * nbt, (NCV + nblk - 1) / nblk);
    const LaunchPlan plan = make_plan("lc_bwd_data_fast", {MT, NT, NCELL, AP, NW, (int)sizeof(T), 0, AP}, {strips, RS, nbt},
                                      grid, 64 * NW, lds);
    if (int rc = check_backward_data_fast(g, plan)) return rc;
    LC_LAUNCH(plan, "lc_backward_data launch", kern, s, g, dy, w, dx, strips, RS, nbt);
    return LC_OK;
}

// The pipelined kernels address a batch tile's dy (64 images) with 32-bit byte offsets.
inline bool pipelined_offsets_fit(const Geom &g) { return (long long)64 * g.L * g.F * 4 < (1LL << 32); }

// The pipelined kernel for filters in blocks of 16 and fields that tile the cells exactly; *done tells whether a
// kernel was launched.  T = float or bf16_t (bf16 storage widened on the way in).
template <typename T>
int launch_backward_data_fast_path(const Geom &g, const T *dy, const T *w, float *dx, hipStream_t s, bool *done) {
    *done = false;
    // pipelined kernel: filters in blocks of 16, fields that tile the cells exactly, a batch tile of 64 images
    if (g.F % 16 == 0 && g.R % g.S == 0 && g.B > 32 && pipelined_offsets_fit(g)) {
        const int ap = g.R / g.S, ntt = (g.S * g.S * g.C + 15) / 16;   // steps per chunk, tiles of 16 cell values
#define LC_BD(AP_, NT_, NCELL_) do { *done = true; return launch_fast<4, NT_, NCELL_, AP_>(g, dy, w, dx, s); } while (0)
        if (ap == 2) {
            if (ntt <= 3) LC_BD(2, 3, 4);
            if (ntt == 4) LC_BD(2, 4, 4);
            LC_BD(2, 3, 1);
        } else if (ap == 3) {
            if (ntt <= 2) LC_BD(3, 2, 4);
            if (ntt == 3) LC_BD(3, 3, 4);
            if (ntt == 4) LC_BD(3, 4, 4);
            LC_BD(3, 4, 2);
        } else if (ap == 4) {
            // wide images: eight cells per workgroup stage 11 field columns instead of 2 x 7 (the paper's first
            // layer: 6.04 -> 5.89 ms); with 5 x 5 covering fields and 50 cells per row the same loses
            // fp32, filters in blocks of 32: whole-line chunks (the paper's first layer: 6.08 -> 5.57 ms)
            if constexpr (sizeof(T) == 4) {
                if (ntt == 3 && g.F % 32 == 0) { *done = true; return launch_line<4, 3, 4, 4, 2>(g, (const float *)dy, (const float *)w, dx, s); }
            }
            if (ntt == 3 && (g.W + g.S - 1) / g.S >= 64) { *done = true; return launch_fast<4, 3, 8, 4, 8>(g, dy, w, dx, s); }
            if (ntt <= 2) LC_BD(4, 2, 4);
            if (ntt == 3) LC_BD(4, 3, 4);
            if (ntt == 4) LC_BD(4, 4, 4);
            LC_BD(4, 4, 2);
        } else if (ap == 5) {
            // fp32, filters in blocks of 32: whole-line chunks (5 x 5 covering fields, 104 x 104 x 12 input, batch 128: 243 -> 233 us;
            // on a 200 x 200 x 3 input under 46 x 46 fields of 32 filters the kernel that loads dy straight into LDS takes
            // 224 us against this one's 220, with 128-image tiles 263 us (two buffers) and 278 us (one); on 64-image
            // tiles with one buffer 229 us at two or three waves per SIMD, with eight cells per workgroup 235 us; with
            // twelve waves (four cells x three tiles of cell values, each wave all 128 images, so that every weight is
            // requested once) 235 us: 650 workgroups, one per compute unit, are three rounds where the work is 2.3.
            // Reading a step's weights as whole lines per quad of lanes (a timing build, the values in the wrong
            // lanes) was no faster either: 229 us.  Nor does the launch lose much to its last, partly filled round of
            // workgroups: with the 1024 workgroups of two whole rounds in one launch (180 us) and the other full-cost
            // pairs and the edge rows in a second one on 32-image tiles (50 us) the layer took 226 us.)
            if constexpr (sizeof(T) == 4) {
                if (ntt <= 3 && g.F % 32 == 0) { *done = true; return launch_line<4, 3, 4, 5, 2>(g, (const float *)dy, (const float *)w, dx, s); }
            }
            if (ntt <= 3) LC_BD(5, 3, 4);
            if (ntt == 4) LC_BD(5, 4, 4);
            LC_BD(5, 4, 2);
        } else if (ap == 8) {
            // one tile of cell values per wave: eight cells per workgroup share the staged fields
            if (ntt == 1) {
                *done = true;
                return launch_fast<4, 1, 8, 8, 8>(g, dy, w, dx, s);
            }
            LC_BD(8, 2, 2);
        }
#undef LC_BD
    }
    return LC_OK;
}

}  // namespace

namespace {

// the masked kernel (any shape), batch tile by batch size
template <typename T>
int launch_backward_data_generic(const Geom &g, const T *dy, const T *w, float *dx, hipStream_t s) {
    if (g.B > 64) return launch_mt<8>(g, dy, w, dx, s);
    if (g.B > 32) return launch_mt<4>(g, dy, w, dx, s);
    if (g.B > 16) return launch_mt<2>(g, dy, w, dx, s);
    return launch_mt<1>(g, dy, w, dx, s);
}

}  // namespace

int launch_backward_data_f32(const Geom &g, const float *dy, const float *w, float *dx, hipStream_t s) {
    // cells of 128-value blocks: one cell per workgroup, dy through LDS, 128 x 128 output tiles
    if (backward_data_wide_supported(g) || backward_data_dense_supported(g))
        return launch_backward_data_wide_f32(g, dy, w, dx, s);
    {
        bool done = false;
        const int rc = launch_backward_data_fast_path(g, dy, w, dx, s, &done);
        if (done) return rc;
    }
    return launch_backward_data_generic(g, dy, w, dx, s);
}

// shapes the pipelined kernel takes (on bf16 storage it multiplies with bf16 matrix instructions)
bool backward_data_bf16_pipelined_supported(const Geom &g) {
    if (!(g.F % 16 == 0 && g.R % g.S == 0 && g.B > 32 && pipelined_offsets_fit(g))) return false;
    const int ap = g.R / g.S;
    return ap == 2 || ap == 3 || ap == 4 || ap == 5 || ap == 8;
}

int launch_backward_data_bf16_storage(const Geom &g, const void *dy, const void *w, float *dx, hipStream_t s) {
    bool done = false;
    const int rc = launch_backward_data_fast_path(g, (const bf16_t *)dy, (const bf16_t *)w, dx, s, &done);
    if (done) return rc;
    return launch_backward_data_generic(g, (const bf16_t *)dy, (const bf16_t *)w, dx, s);
}

}  // namespace lc
