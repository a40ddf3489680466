// lc_backward_weights: out[l,k,f] = beta*out[l,k,f] + gamma * sum_p sum_b patch(x_p)[b,l,k] * dy_p[b,l,f]
// (the weight gradient of Eq. 1; two operand pairs because the tied weights are used twice).
//
// The contraction runs over the batch, so both MFMA operands are read straight from global memory
// with lanes along the contiguous axis: A[k][b] lanes run along k (the (kw,c) run of an image row),
// B[b][f] lanes run along f.  Waves are independent: each owns one location, MTW tiles of 16 patch
// elements and NT tiles of 16 filters, loops over the batch four images at a time and writes its
// MTW x NT output tiles once.
#include <type_traits>
#include "lc_common.hpp"

namespace lc {

// T: storage type of x and dy (float, or bf16 bit patterns widened on their way in).
template <int MTW, int NT, typename T, bool SSQ>
__global__ __launch_bounds__(256) void lc_bwd_weights_kernel(Geom g, const T *__restrict__ x1,
                                                             const T *__restrict__ dy1,
                                                             const T *__restrict__ x2,
                                                             const T *__restrict__ dy2, float beta, float gamma,
                                                             float *__restrict__ out, float *__restrict__ ssq,
                                                             int kblocks, int ntasks) {
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
        const T *x = p ? x2 : x1;
        const T *dy = p ? dy2 : dy1;
        if (!x) break;
        const T *xa = x + (size_t)kk * img;
        const T *da = dy + ((size_t)kk * g.L + loc) * g.F + f0 + m;
        const size_t dstep = (size_t)g.L * g.F;
        if (!edge) {
#pragma unroll 2
            for (int b0 = 0; b0 < Bfull; b0 += 4) {
                float a[MTW], bv[NT];
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt) a[mt] = ld_f32(xa + (size_t)b0 * img + off[mt]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) bv[nt] = ld_f32(da + (size_t)b0 * dstep + nt * 16);
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
            for (int mt = 0; mt < MTW; ++mt) a[mt] = (bok && kok[mt]) ? ld_f32(xa + (size_t)b0 * img + off[mt]) : 0.f;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) bv[nt] = (bok && fok[nt]) ? ld_f32(da + (size_t)b0 * dstep + nt * 16) : 0.f;
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = mfma16(a[mt], bv[nt], acc[mt][nt]);
        }
    }

    float *ol = out + (size_t)loc * g.K * g.F;
    float sq[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) sq[nt] = 0.f;
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
                float v = gamma * acc[mt][nt][r];
                if (beta != 0.f) v += beta * *o;
                *o = v;
                if (SSQ) sq[nt] += v * v;
            }
        }
    // per-filter sums of squares of the rows this wave stored: partial [location][k block][filter]
    if (SSQ) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float t = sq[nt];
            t += __shfl_xor(t, 16, 64);
            t += __shfl_xor(t, 32, 64);
            if (kk == 0 && fok[nt]) ssq[((size_t)loc * kblocks + (k0 / (MTW * 16))) * g.F + f0 + nt * 16 + m] = t;
        }
    }
}


// ---------------------------------------------------------------------------------------------
// Fast path (aligned shapes).  Same decomposition, but every global access covers whole cache
// lines, by permuting which rows/columns of the MFMA tiles a lane owns:
//   A: lane (m,kk) loads VA consecutive patch elements k = kg + VA*m .. +VA-1 of image b0+kk in one
//      dwordxVA load; element t of that vector is row m of M-tile t (tile t holds k = kg + VA*m + t).
//      16 lanes x VA floats are contiguous in the image row.
//   B: lane (n,kk) loads NT consecutive filters f = f0 + NT*n .. of image b0+kk; element u is column
//      n of N-tile u.  16 lanes x NT floats are contiguous in dy.
//   D: lane (n, 4*(l/16)+r) of tile (t,u) is out[k = kg + VA*(4*(l/16)+r) + t][f0 + NT*n + u]: the
//      NT tiles of one row are stored as one dwordxNT, 16 lanes covering a contiguous run of w.
// Loads run PF batch steps ahead of the MFMAs in a register ring.
template <int N> struct VecT;
template <> struct VecT<1> { typedef float T; };
template <> struct VecT<2> { typedef float T __attribute__((ext_vector_type(2))); };
template <> struct VecT<4> { typedef float T __attribute__((ext_vector_type(4))); };

template <int N>
__device__ __forceinline__ float vget(const typename VecT<N>::T &v, int i) {
    if constexpr (N == 1) return v; else return v[i];
}

// SSQ: also leave, per location, block of patch elements and filter, the sum of squares of the values stored (a
// code path of its own: the plain weight gradient carries none of it).
template <int G, int VA, int NT, int PF, typename T = float, bool SSQ = false>
// More waves per SIMD than the registers give by themselves do not pay: with 32 filters and blocks of 128 patch
// elements, bounds of three and four waves per SIMD took 242 and 248-290 us against 221 us at two (the loads of
// more waves in flight evict each other's lines from the vector cache).
__global__ __launch_bounds__(256, G == 3 ? 2 : 1) void lc_bwd_weights_fast_kernel(Geom g, const T *__restrict__ x1,
                                                                  const T *__restrict__ dy1,
                                                                  const T *__restrict__ x2,
                                                                  const T *__restrict__ dy2, float beta,
                                                                  float gamma, float *__restrict__ out,
                                                                  float *__restrict__ ssq, int kblocks, int ntasks) {
    typedef typename RawVec<T, VA>::V AV;     // VA consecutive patch elements as loaded (fp32, or bf16 bit patterns)
    typedef typename RawVec<T, NT>::V BR;     // NT consecutive dy values as loaded
    typedef typename VecT<NT>::T BV;          // NT consecutive outputs
    // global address space: plain global_load, not flat.  The patch vectors are only element-aligned in general
    // (a field starts every S*C elements): the declared alignment says so, and the vector load stays one instruction
    typedef __attribute__((address_space(1), aligned(sizeof(T)))) AV GAV;
    typedef __attribute__((address_space(1))) BR GBV;
    typedef const __attribute__((address_space(1))) T *gfloat_ptr;
    constexpr int KB = G * VA * 16;  // patch elements per task
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, kk = lane >> 4;
    const int task = remap_xcd(blockIdx.x, gridDim.x) * 4 + wave;
    if (task >= ntasks) return;
    // Where a wave loads more of x than of dy per batch step (G * VA > NT), tasks are ordered field row by field row,
    // inside a row block of patch elements by block, and the fields of the row innermost: the four waves of a
    // workgroup, and the workgroups next to it on the same XCD, then read the same image rows at the same time
    // (horizontally adjacent fields share (R-S)/R of their patch rows), and what one of them fetched the others find
    // in the caches (K = 1200, 32 filters, 46 fields per row, batch 128: 219 -> 201 us).  Otherwise the blocks of a
    // field are innermost and the waves of a workgroup share the field's dy (16 x 16 x 3 patches, 384 filters in
    // tiles of 64: 4.90 ms against 4.98 ms in the other order).  Ordering the tasks so that vertically adjacent
    // fields' blocks over the same image rows also run together (blocks 2 i + kb in turn) took 323 us; workgroups of
    // two, eight and sixteen waves instead of four 207, 218 and 239 us.
    int loc, k0;
    if constexpr (G * VA > NT) {
        const int per_row = g.LW * kblocks;
        const int i = task / per_row, rr = task - i * per_row;
        const int kb = rr / g.LW;
        loc = i * g.LW + (rr - kb * g.LW);
        k0 = kb * KB;
    } else {
        loc = task / kblocks;
        k0 = (task - loc * kblocks) * KB;
    }
    const int i = loc / g.LW, j = loc - i * g.LW;
    const int f0 = blockIdx.y * NT * 16;
    const size_t img = (size_t)g.H * g.W * g.C;

    // Rows of the A tiles that fall beyond K are loaded from a valid address (element 0 of the patch)
    // and never masked: row m of A only reaches row m of D, and those rows are not stored.
    int off[G];
#pragma unroll
    for (int gg = 0; gg < G; ++gg) {
        const int k = k0 + gg * VA * 16 + VA * m;
        const int kc = k < g.K ? k : 0;
        const int kh = kc / g.RC, rem = kc - kh * g.RC;
        off[gg] = ((i * g.S + kh) * g.W + j * g.S) * g.C + rem;
    }

    f32x4 acc[G][VA][NT];
#pragma unroll
    for (int gg = 0; gg < G; ++gg)
#pragma unroll
        for (int t = 0; t < VA; ++t)
#pragma unroll
            for (int u = 0; u < NT; ++u) acc[gg][t][u] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int nsteps = g.B >> 2;                 // B % (4*PF) == 0 on this path
    const size_t xstep = 4 * img, dstep = (size_t)4 * g.L * g.F;
    // The last block of a field may reach K before its G groups of VA tiles are used up (K = 1200 in blocks of 128:
    // the tenth block holds 48 elements, one group).  Groups that lie wholly beyond K are neither loaded nor
    // multiplied: GA of the G groups are live, the same for the whole wave.
    auto contract = [&](auto ga_tag) {
        constexpr int GA = decltype(ga_tag)::value;
        for (int p = 0; p < 2; ++p) {
            const T *x = p ? x2 : x1;
            const T *dy = p ? dy2 : dy1;
            if (!x) break;
            gfloat_ptr xa[GA];
#pragma unroll
            for (int gg = 0; gg < GA; ++gg) xa[gg] = (gfloat_ptr)x + ((size_t)kk * img + off[gg]);
            gfloat_ptr da = (gfloat_ptr)dy + (((size_t)kk * g.L + loc) * g.F + f0 + NT * m);
            AV a[PF][GA];
            BR bv[PF];
            // ring prologue: steps 0 .. PF-1
#pragma unroll
            for (int ss = 0; ss < PF; ++ss) {
#pragma unroll
                for (int gg = 0; gg < GA; ++gg) { a[ss][gg] = *(const GAV *)xa[gg]; xa[gg] += xstep; }
                bv[ss] = *(const GBV *)da; da += dstep;
            }
            // steady state: consume slot ss, then refill it with step s+PF
            for (int s0 = PF; s0 < nsteps; s0 += PF) {
#pragma unroll
                for (int ss = 0; ss < PF; ++ss) {
#pragma unroll
                    for (int gg = 0; gg < GA; ++gg)
#pragma unroll
                        for (int t = 0; t < VA; ++t)
#pragma unroll
                            for (int u = 0; u < NT; ++u)
                                acc[gg][t][u] = mfma16(raw_get<T, VA>(a[ss][gg], t), raw_get<T, NT>(bv[ss], u), acc[gg][t][u]);
#pragma unroll
                    for (int gg = 0; gg < GA; ++gg) { a[ss][gg] = *(const GAV *)xa[gg]; xa[gg] += xstep; }
                    bv[ss] = *(const GBV *)da; da += dstep;
                    // keep the refill of slot ss right behind the MFMAs that consumed it: the loads then run
                    // PF-1 slots ahead of their use instead of being sunk to the end of the iteration
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // drain
#pragma unroll
            for (int ss = 0; ss < PF; ++ss)
#pragma unroll
                for (int gg = 0; gg < GA; ++gg)
#pragma unroll
                    for (int t = 0; t < VA; ++t)
#pragma unroll
                        for (int u = 0; u < NT; ++u)
                            acc[gg][t][u] = mfma16(raw_get<T, VA>(a[ss][gg], t), raw_get<T, NT>(bv[ss], u), acc[gg][t][u]);
        }
    };
    const int ga = min(G, (g.K - k0 + VA * 16 - 1) / (VA * 16));
    if constexpr (G == 1) {
        contract(std::integral_constant<int, 1>{});
    } else if constexpr (G == 2) {
        if (ga == 2) contract(std::integral_constant<int, 2>{});
        else contract(std::integral_constant<int, 1>{});
    } else if constexpr (G == 3) {
        if (ga == 3) contract(std::integral_constant<int, 3>{});
        else if (ga == 2) contract(std::integral_constant<int, 2>{});
        else contract(std::integral_constant<int, 1>{});
    } else {
        static_assert(G == 4, "groups per block");
        if (ga == 4) contract(std::integral_constant<int, 4>{});
        else if (ga == 3) contract(std::integral_constant<int, 3>{});
        else if (ga == 2) contract(std::integral_constant<int, 2>{});
        else contract(std::integral_constant<int, 1>{});
    }

    float *ol = out + (size_t)loc * g.K * g.F + f0 + NT * m;
    // per-filter sums of squares of the rows this wave stores (only formed when ssq is given)
    float sq[NT];
#pragma unroll
    for (int u = 0; u < NT; ++u) sq[u] = 0.f;
    auto add_squares = [&](const BV &v) {
        if constexpr (NT == 1) {
            sq[0] += v * v;
        } else {
#pragma unroll
            for (int u = 0; u < NT; ++u) sq[u] += v[u] * v[u];
        }
    };
    auto store_squares = [&]() {
#pragma unroll
        for (int u = 0; u < NT; ++u) {
            sq[u] += __shfl_xor(sq[u], 16, 64);
            sq[u] += __shfl_xor(sq[u], 32, 64);
        }
        if (kk == 0) {
            BV t;
            if constexpr (NT == 1) {
                t = sq[0];
            } else {
#pragma unroll
                for (int u = 0; u < NT; ++u) t[u] = sq[u];
            }
            *(BV *)(ssq + ((size_t)loc * kblocks + (k0 / KB)) * g.F + f0 + NT * m) = t;
        }
    };
    if (beta == 0.f) {
#pragma unroll
        for (int gg = 0; gg < G; ++gg)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int t = 0; t < VA; ++t) {
                    const int k = k0 + gg * VA * 16 + VA * (4 * kk + r) + t;
                    if (k >= g.K) continue;
                    BV v;
                    if constexpr (NT == 1) {
                        v = gamma * acc[gg][t][0][r];
                    } else {
#pragma unroll
                        for (int u = 0; u < NT; ++u) v[u] = gamma * acc[gg][t][u][r];
                    }
                    *(BV *)(ol + (size_t)k * g.F) = v;
                    if constexpr (SSQ) add_squares(v);
                }
        if constexpr (SSQ) store_squares();
        return;
    }
    // beta != 0 (the fused update), a code path of its own: the old values of four rows are requested together,
    // before the first is used.  A load under its own condition in front of each store makes the compiler wait
    // for it on the spot: one round trip to memory per row, 32 of them in a row.  (All 16 or 32 rows at once cost
    // the registers of a wave per SIMD on the narrow layers.)  Rows beyond K read row 0 instead and are not stored.
#pragma unroll
    for (int gg = 0; gg < G; ++gg)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            BV old[VA];
#pragma unroll
            for (int t = 0; t < VA; ++t) {
                const int k = k0 + gg * VA * 16 + VA * (4 * kk + r) + t;
                old[t] = *(const BV *)(ol + (size_t)(k < g.K ? k : 0) * g.F);
            }
#pragma unroll
            for (int t = 0; t < VA; ++t) {
                const int k = k0 + gg * VA * 16 + VA * (4 * kk + r) + t;
                if (k >= g.K) continue;
                BV v;
                if constexpr (NT == 1) {
                    v = gamma * acc[gg][t][0][r];
                } else {
#pragma unroll
                    for (int u = 0; u < NT; ++u) v[u] = gamma * acc[gg][t][u][r];
                }
                v += beta * old[t];
                *(BV *)(ol + (size_t)k * g.F) = v;
                if constexpr (SSQ) add_squares(v);
            }
        }
    if constexpr (SSQ) store_squares();
}

namespace {

// Host check of a lc_bwd_weights_kernel launch.  tparam = {MTW, NT, bytes per operand element}; arg = {blocks of 16*MTW patch elements per
// field, wave tasks}.  The kernel masks every ragged edge itself.
int check_backward_weights_generic(const Geom &g, const LaunchPlan &p) {
    const int MTW = p.tparam[0], NT = p.tparam[1];
    const int kblocks = p.arg[0], ntasks = p.arg[1];
    LC_PLAN_REQUIRE(p, p.block == 256);
    LC_PLAN_REQUIRE(p, kblocks == ceil_div(g.K, 16 * MTW) && (long long)ntasks == (long long)g.L * kblocks);
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] * 4 >= ntasks && (long long)(p.grid[0] - 1) * 4 < ntasks);
    LC_PLAN_REQUIRE(p, (long long)p.grid[1] * NT * 16 >= g.F && (long long)(p.grid[1] - 1) * NT * 16 < g.F && p.grid[2] == 1);
    return LC_OK;
}

template <int MTW, int NT, typename T>
int launch_one(const Geom &g, const T *x1, const T *dy1, const T *x2, const T *dy2, float beta,
               float gamma, float *out, float *ssq, int *kblocks_out, hipStream_t s) {
    const int kt = (g.K + 15) / 16;
    const int kblocks = (kt + MTW - 1) / MTW;
    const long long ntasks = (long long)g.L * kblocks;
    if (ntasks > (1LL << 30)) return LC_EUNSUPPORTED;
    dim3 grid((unsigned)((ntasks + 3) / 4), (g.F + NT * 16 - 1) / (NT * 16));
    const LaunchPlan plan = make_plan("lc_bwd_weights_generic", {MTW, NT, (int)sizeof(T)}, {kblocks, (int)ntasks}, grid, 256, 0);
    if (int rc = check_backward_weights_generic(g, plan)) return rc;
    if (kblocks_out) *kblocks_out = kblocks;
    if (ssq)
        LC_LAUNCH(plan, "lc_backward_weights launch", (lc_bwd_weights_kernel<MTW, NT, T, true>), s, g, x1, dy1, x2, dy2,
                  beta, gamma, out, ssq, kblocks, (int)ntasks);
    else
        LC_LAUNCH(plan, "lc_backward_weights launch", (lc_bwd_weights_kernel<MTW, NT, T, false>), s, g, x1, dy1, x2, dy2,
                  beta, gamma, out, ssq, kblocks, (int)ntasks);
    return LC_OK;
}

template <int NT, typename T>
int launch_nt(const Geom &g, const T *x1, const T *dy1, const T *x2, const T *dy2, float beta,
              float gamma, float *out, float *ssq, int *kblocks_out, hipStream_t s) {
    // tiles of 16 patch elements per wave: the candidate with the least padding of K, larger first
    const int kt = (g.K + 15) / 16;
    const int cand[4] = {8, 6, 5, 4};
    int best = 8, waste = 1 << 30;
    for (int c : cand) {
        const int wst = (kt + c - 1) / c * c - kt;
        if (wst < waste) { waste = wst; best = c; }
    }
    switch (best) {
        case 8: return launch_one<8, NT>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
        case 6: return launch_one<6, NT>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
        case 5: return launch_one<5, NT>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
        default: return launch_one<4, NT>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
    }
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Layers with one tile of 16 filters per field (fp32, a batch of 4*NB images that fits LDS whole).  The kernels above
// give a wave one block of patch elements of one field and let it fetch its operands itself: every x element is used
// for 16 filters only, eight MFMA flops per byte fetched, and the caches cannot keep up.  Here a workgroup is a strip
// of eight fields of one field row, one field per wave, as in the forward kernels:
//   - a chunk is one patch row of the strip for the whole batch, loaded from global memory straight into LDS (16
//     bytes per lane; lane i of a wave's load lands 16 i bytes past the load's LDS base), two buffers, the next
//     chunk in flight while this one is multiplied; the loads are inline assembly and the waits on them are written
//     out (the memory counter counts loads and stores in program order: behind a chunk's x loads come only the
//     stores, and for beta != 0 the loads, of the previous chunk's epilogue, a number known at compile time);
//   - a wave's B operands, dy of its field for the whole batch (one float per lane and batch step of four images),
//     are loaded once and stay in registers for all R chunks, for both terms;
//   - the A operand of batch step s and tile t, lane (m,kk), is x[4s+kk][16t+m] of the field's window in the
//     staged strip: one 4-byte LDS read per MFMA at a compile-time offset from one address register; the LDS row
//     stride is 16 or 48 floats past a multiple of 64, so the 16 x 4 floats of a read cover all 64 banks;
//   - a chunk's MTR tiles (16*MTR rows of dW) are finished after the batch has been summed over for both terms
//     and are stored (or merged into the old weights) before the next chunk starts.
// Images, strips and fields at the ragged end: waves past the last field of the row shadow that field and store
// nothing; vectors past the image row are clamped into it and only reach those waves.
template <int NLOC, int MTR, int NB, int NSLOT, int RV, bool SSQ>
__global__ __launch_bounds__(64 * NLOC, NLOC == 8 ? 2 : 1) void lc_bwd_weights_strip_kernel(
    Geom g, const float *__restrict__ x1, const float *__restrict__ dy1, const float *__restrict__ x2,
    const float *__restrict__ dy2, float beta, float gamma, float *__restrict__ out, float *__restrict__ ssq,
    int strips_per_row, int sq4) {
    constexpr int NTHR = 64 * NLOC, RS = RV * 4, BT = 4 * NB, BUF = NSLOT * NTHR * 4;
    constexpr int NG = NB / 2;                // batch steps are read from LDS in groups of two
    static_assert(NB % 16 == 0 && NSLOT <= NG / 2, "one x load per group in the first half of a chunk's groups");
    static_assert((4 * (NB / 2 - 1) * RS + 16 * (MTR - 1)) * 4 < 65536, "LDS read offsets are 16-bit immediates");
    extern __shared__ __attribute__((aligned(16))) float xs[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 15, kk = lane >> 4;
    const int work = remap_xcd(blockIdx.x, gridDim.x);
    const int i = work / strips_per_row, j0 = (work - i * strips_per_row) * NLOC;
    const int j = j0 + wave;
    const bool active = j < g.LW;
    const int loc = i * g.LW + (active ? j : g.LW - 1);
    const int f0 = blockIdx.y * 16;
    const int SC = g.S * g.C, WC = g.W * g.C;
    const size_t img = (size_t)g.H * WC;
    const int col0 = j0 * SC;
    const bool two = x2 != nullptr;

    // B operands: dy[4s+kk][loc][f0+m] for every batch step s, of both terms
    float dyr[2][NB];
    {
        const float *d1 = dy1 + ((size_t)kk * g.L + loc) * g.F + f0 + m;
        const float *d2 = (two ? dy2 : dy1) + ((size_t)kk * g.L + loc) * g.F + f0 + m;
        const size_t dstep = (size_t)4 * g.L * g.F;
#pragma unroll
        for (int s = 0; s < NB; ++s) {
            dyr[0][s] = d1[s * dstep];
            dyr[1][s] = d2[s * dstep];
        }
    }

    // where this lane's vector of load q comes from: bytes past the chunk's first vector (image 0, image row
    // i*S + kh, column col0); pad vectors and the slack behind the last row load that first vector
    unsigned goff[NSLOT];
    {
        const int lim = WC - col0 - 4;
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            const int P = q * NTHR + tid, b = P / RV, v = P - b * RV;
            const bool data = b < BT && v < sq4;
            goff[q] = data ? (unsigned)(((size_t)b * img + min(4 * v, max(lim, 0))) * 4) : 0u;
        }
    }
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) float *)xs + wave * 64 * 16;

    const float *abase = xs + kk * RS + wave * SC + m;
    f32x4 acc[MTR];
    // The rows of out a chunk finishes: kh*RC + 16t + 4kk + r.  The address is a scalar base (field, chunk, row) plus
    // the lane's offset, so the epilogue has no address arithmetic in vector registers.
    const unsigned olane = (unsigned)((4 * kk * g.F + m) * 4);
    auto out_row = [&](int kh, int t, int r) -> gbyte_ptr {
        return (gbyte_ptr)(out + ((size_t)loc * g.K + (size_t)kh * g.RC + 16 * t + r) * g.F + f0);
    };
    float old[MTR][4];      // beta != 0: the rows' old values, requested at the start of the chunk's last term

    // Batch steps of one chunk and term out of LDS buffer buf: groups of two steps, the next group's reads issued
    // behind the first MFMAs of the current one.  The x loads of the chunk-term after this one (row kh_next of
    // src_next, into the other buffer) go out one per group over the first groups: issued all at once at the
    // chunk's start they queue up in the compute unit's one address unit (16 cycles per load) and the waves, which
    // issue in order, stand behind them before their first MFMA; in the first half, so that the last one has half a
    // chunk to land.
    auto contract = [&](int term, int buf, const float *src_next, int kh_next) {
        gbyte_ptr nbase = (gbyte_ptr)(src_next + (size_t)(i * g.S + kh_next) * WC + col0);
        const unsigned nl = lds0 + (buf ^ 1) * (BUF * 4);
        const float *ar = abase + buf * BUF;
        const float *ar2 = ar + 4 * (NB / 2) * RS;        // second half of the batch (16-bit read offsets)
        float a[2][2][MTR];
        auto read_group = [&](int gs, float (&dst)[2][MTR]) {
#pragma unroll
            for (int ss = 0; ss < 2; ++ss)
#pragma unroll
                for (int t = 0; t < MTR; ++t) {
                    const int s = 2 * gs + ss;
                    dst[ss][t] = s < NB / 2 ? ar[4 * s * RS + 16 * t] : ar2[4 * (s - NB / 2) * RS + 16 * t];
                }
        };
        read_group(0, a[0]);
#pragma unroll
        for (int gs = 0; gs < NG; ++gs) {
#pragma unroll
            for (int ss = 0; ss < 2; ++ss) {
#pragma unroll
                for (int t = 0; t < MTR; ++t)
                    acc[t] = mfma16(a[gs & 1][ss][t], dyr[term][2 * gs + ss], acc[t]);
                __builtin_amdgcn_sched_barrier(0);
                if (ss == 0) {
                    if (gs + 1 < NG) read_group(gs + 1, a[(gs + 1) & 1]);
                    if (gs < NSLOT) load_lds16(nbase, goff[gs], nl + gs * (NTHR * 16));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };
    float sq = 0.f;      // sum of squares of the values this lane stored (one filter: f0 + m)

    // initial chunk: all its x loads at once
    {
        gbyte_ptr base = (gbyte_ptr)(x1 + (size_t)(i * g.S) * WC + col0);
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) load_lds16(base, goff[q], lds0 + q * (NTHR * 16));
    }
    wait_loads<0>();
    // The compiler's own wait insertion must see the dy loads finished here: otherwise it keeps waiting for them
    // inside the loop, by counts that know nothing of the x loads in flight there and so wait for those as well.
#pragma unroll
    for (int s = 0; s < NB; ++s) {
        asm volatile("" : "+v"(dyr[0][s]));
        asm volatile("" : "+v"(dyr[1][s]));
    }
    __syncthreads();
    int u = 0;       // chunk-terms done: the buffer in use is u & 1
    for (int kh = 0; kh < g.R; ++kh) {
        const int khn = kh + 1 < g.R ? kh + 1 : kh;      // the last chunk loads itself once more (values unused)
#pragma unroll
        for (int t = 0; t < MTR; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
        if (two) {
            contract(0, u & 1, x2, kh);
            wait_loads<0>();      // nothing was issued behind the x loads
            __syncthreads();
            ++u;
        }
        // The chunk's last term.  Memory operations of this wave from here to the barrier, in order: the rows' old
        // values (4*MTR loads; beta != 0 and the wave stores at all), the NSLOT x loads of the next chunk-term, the
        // 4*MTR stores of the epilogue.  The old values are waited for with the x loads still in flight, and the
        // barrier with the stores still in flight.
        const bool merge = active && beta != 0.f;
        if (merge) {
#pragma unroll
            for (int t = 0; t < MTR; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) old[t][r] = load_nowait<1>(out_row(kh, t, r), olane);
        }
        contract(two ? 1 : 0, u & 1, x1, khn);
        if (active) {
            if (merge) {
#pragma unroll
                for (int t = 0; t < MTR; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) wait_loads<NSLOT>(old[t][r]);
            }
#pragma unroll
            for (int t = 0; t < MTR; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float v = merge ? gamma * acc[t][r] + beta * old[t][r] : gamma * acc[t][r];
                    store_nowait(out_row(kh, t, r), olane, v);
                    if constexpr (SSQ) sq += v * v;
                }
            wait_loads<4 * MTR>();      // the x loads of the next chunk-term have landed; the stores may fly on
        } else {
            wait_loads<0>();
        }
        __syncthreads();
        ++u;
    }
    if constexpr (SSQ) {
        // per filter: lanes (m, kk = 0..3) hold the partial sums of the filter's rows; one partial per field
        sq += __shfl_xor(sq, 16, 64);
        sq += __shfl_xor(sq, 32, 64);
        if (active && kk == 0) ssq[(size_t)loc * g.F + f0 + m] = sq;
    }
}

namespace {

// Host check of a lc_bwd_weights_fast_kernel launch.  tparam = {G, VA, NT, PF, bytes per operand element};
// arg = {blocks of G*VA*16 patch elements per field, wave tasks}.
int check_backward_weights_fast(const Geom &g, const LaunchPlan &p) {
    const int G = p.tparam[0], VA = p.tparam[1], NT = p.tparam[2], PF = p.tparam[3];
    const int kblocks = p.arg[0], ntasks = p.arg[1];
    const int KB = G * VA * 16;
    LC_PLAN_REQUIRE(p, p.block == 256 && (VA == 1 || VA == 2 || VA == 4) && (NT == 1 || NT == 2 || NT == 4));
    // a lane's VA patch elements never straddle two patch rows; filters in whole tiles
    LC_PLAN_REQUIRE(p, g.RC % VA == 0 && g.F % (NT * 16) == 0 && (int)p.grid[1] == g.F / (NT * 16) && p.grid[2] == 1);
    // the batch in whole ring turns of PF steps of four images
    LC_PLAN_REQUIRE(p, PF >= 1 && g.B % (4 * PF) == 0);
    LC_PLAN_REQUIRE(p, kblocks == ceil_div(g.K, KB) && (long long)ntasks == (long long)g.L * kblocks);
    LC_PLAN_REQUIRE(p, (long long)p.grid[0] * 4 >= ntasks && (long long)(p.grid[0] - 1) * 4 < ntasks);
    // 32-bit offsets inside one image
    LC_PLAN_REQUIRE(p, (long long)g.H * g.W * g.C < (1LL << 31));
    return LC_OK;
}

template <int G, int VA, int NT, int PF, typename T>
int launch_fast(const Geom &g, const T *x1, const T *dy1, const T *x2, const T *dy2, float beta,
                float gamma, float *out, float *ssq, int *kblocks_out, hipStream_t s) {
    constexpr int KB = G * VA * 16;
    const int kblocks = (g.K + KB - 1) / KB;
    const long long ntasks = (long long)g.L * kblocks;
    if (ntasks > (1LL << 30)) return LC_EUNSUPPORTED;
    dim3 grid((unsigned)((ntasks + 3) / 4), g.F / (NT * 16));
    const LaunchPlan plan = make_plan("lc_bwd_weights_fast", {G, VA, NT, PF, (int)sizeof(T)}, {kblocks, (int)ntasks}, grid, 256, 0);
    if (int rc = check_backward_weights_fast(g, plan)) return rc;
    if (kblocks_out) *kblocks_out = kblocks;
    if (ssq)
        LC_LAUNCH(plan, "lc_backward_weights launch", (lc_bwd_weights_fast_kernel<G, VA, NT, PF, T, true>), s, g, x1, dy1,
                  x2, dy2, beta, gamma, out, ssq, kblocks, (int)ntasks);
    else
        LC_LAUNCH(plan, "lc_backward_weights launch", (lc_bwd_weights_fast_kernel<G, VA, NT, PF, T, false>), s, g, x1, dy1,
                  x2, dy2, beta, gamma, out, ssq, kblocks, (int)ntasks);
    return LC_OK;
}

// Host check of a lc_bwd_weights_strip_kernel launch.  tparam = {MTR, NB, NSLOT, RV, NLOC}; arg = {strips per field row,
// sq4}.
int check_backward_weights_strip(const Geom &g, const LaunchPlan &p) {
    const int MTR = p.tparam[0], NB = p.tparam[1], NSLOT = p.tparam[2], RV = p.tparam[3], NLOC = p.tparam[4];
    const int strips = p.arg[0], sq4 = p.arg[1];
    const int SC = g.S * g.C, WC = g.W * g.C, NTHR = 64 * NLOC;
    LC_PLAN_REQUIRE(p, (NLOC == 8 || NLOC == 16) && (int)p.block == NTHR);
    // the whole batch per chunk; a patch row in whole tiles of 16; filters in whole tiles
    LC_PLAN_REQUIRE(p, g.B == 4 * NB && NB % 16 == 0 && g.RC == 16 * MTR && g.F % 16 == 0);
    LC_PLAN_REQUIRE(p, (int)p.grid[1] == g.F / 16 && p.grid[2] == 1);
    LC_PLAN_REQUIRE(p, strips == ceil_div(g.LW, NLOC) && (long long)p.grid[0] == (long long)strips * g.LH);
    // 16-byte vectors of x from every strip's start; the staged strip covers the NLOC windows and fits an LDS row
    LC_PLAN_REQUIRE(p, WC % 4 == 0 && (NLOC * SC) % 4 == 0 && 4 * sq4 >= g.RC + (NLOC - 1) * SC && sq4 <= RV);
    // the 64 floats of an LDS read (16 consecutive ones of four rows) fall into 64 banks
    LC_PLAN_REQUIRE(p, (4 * RV) % 64 == 16 || (4 * RV) % 64 == 48);
    LC_PLAN_REQUIRE(p, (long long)NSLOT * NTHR >= (long long)g.B * RV && p.lds_bytes >= (size_t)2 * NSLOT * NTHR * 16);
    // LDS read offsets (half the batch per base register) are 16-bit immediates; one x load per group of two batch
    // steps in the first half of a chunk; the kernel's waits count at most 4*MTR + NSLOT loads and stores
    LC_PLAN_REQUIRE(p, (4 * (NB / 2 - 1) * 4 * RV + 16 * (MTR - 1)) * 4 < 65536 && NSLOT <= NB / 4 && 4 * MTR + NSLOT <= 63);
    // 32-bit byte offsets into x and into a field's K x F block of out; clamped vectors stay inside the image row
    LC_PLAN_REQUIRE(p, (long long)g.B * g.H * g.W * g.C * 4 < (1LL << 32) && (long long)g.K * g.F * 4 < (1LL << 31) &&
                           WC - (strips - 1) * NLOC * SC >= 4);
    return LC_OK;
}

template <int NLOC, int MTR, int NB, int NSLOT, int RV>
bool backward_weights_strip_fits(const Geom &g) {
    const int SC = g.S * g.C, WC = g.W * g.C, strips = (g.LW + NLOC - 1) / NLOC;
    const int sq4 = ((g.RC + (NLOC - 1) * SC + 3) & ~3) / 4;
    return g.B == 4 * NB && g.RC == 16 * MTR && g.F == 16 && WC % 4 == 0 && (NLOC * SC) % 4 == 0 && sq4 <= RV &&
           (g.B * RV + 64 * NLOC - 1) / (64 * NLOC) <= NSLOT && (long long)g.B * g.H * g.W * g.C * 4 < (1LL << 32) &&
           WC - (strips - 1) * NLOC * SC >= 4;
}

template <int NLOC, int MTR, int NB, int NSLOT, int RV>
int launch_strip(const Geom &g, const float *x1, const float *dy1, const float *x2, const float *dy2, float beta,
                 float gamma, float *out, float *ssq, int *kblocks_out, hipStream_t s) {
    const int strips = (g.LW + NLOC - 1) / NLOC;
    const int sq4 = ((g.RC + (NLOC - 1) * g.S * g.C + 3) & ~3) / 4;
    const size_t lds = (size_t)2 * NSLOT * 64 * NLOC * 16;
    dim3 grid(strips * g.LH, g.F / 16);
    const LaunchPlan plan = make_plan("lc_bwd_weights_strip", {MTR, NB, NSLOT, RV, NLOC}, {strips, sq4}, grid, 64 * NLOC, lds);
    if (int rc = check_backward_weights_strip(g, plan)) return rc;
    if (kblocks_out) *kblocks_out = 1;       // one partial sum of squares per field and filter
    if (ssq)
        LC_LAUNCH(plan, "lc_backward_weights launch", (lc_bwd_weights_strip_kernel<NLOC, MTR, NB, NSLOT, RV, true>), s, g, x1,
                  dy1, x2, dy2, beta, gamma, out, ssq, strips, sq4);
    else
        LC_LAUNCH(plan, "lc_backward_weights launch", (lc_bwd_weights_strip_kernel<NLOC, MTR, NB, NSLOT, RV, false>), s, g, x1,
                  dy1, x2, dy2, beta, gamma, out, ssq, strips, sq4);
    return LC_OK;
}

// widest vector (4, 2, 1 floats) that never straddles two patch rows
int patch_vector_width(const Geom &g) {
    for (int v = 4; v > 1; v >>= 1)
        if (g.RC % v == 0) return v;
    return 1;
}

template <int G, int VA, int NT, typename T>
int launch_fast_pf(const Geom &g, const T *x1, const T *dy1, const T *x2, const T *dy2, float beta,
                   float gamma, float *out, float *ssq, int *kblocks_out, hipStream_t s) {
    if (g.B % 16 == 0) return launch_fast<G, VA, NT, 4>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
    if (g.B % 8 == 0) return launch_fast<G, VA, NT, 2>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
    return launch_fast<G, VA, NT, 1>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
}

// The whole-line kernel for aligned shapes; *done tells whether a kernel was launched.  T = float or bf16_t.
template <typename T>
int launch_backward_weights_fast_path(const Geom &g, const T *x1, const T *dy1, const T *x2, const T *dy2, float beta,
                                      float gamma, float *out, float *ssq, int *kblocks_out, hipStream_t s, bool *done) {
    *done = false;
    if constexpr (sizeof(T) == 4) {
        // 16 filters per field, a batch of 128, patch rows of 48 elements: strips of eight fields out of LDS
        // sixteen fields per workgroup (four waves per SIMD) where that idles no more waves at the end of a field
        // row than eight do
        if ((g.LW + 15) / 16 * 2 == (g.LW + 7) / 8 && backward_weights_strip_fits<16, 3, 32, 5, 36>(g)) {
            *done = true;
            return launch_strip<16, 3, 32, 5, 36>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
        }
        if (backward_weights_strip_fits<8, 3, 32, 7, 28>(g)) {
            *done = true;
            return launch_strip<8, 3, 32, 7, 28>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
        }
    }
    const int va = patch_vector_width(g);
    if ((g.B & 3) == 0 && va == 4) {
        if (g.F % 64 == 0) { *done = true; return launch_fast_pf<1, 4, 4>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s); }
        if (g.F % 32 == 0) {
            *done = true;
            // blocks of 192 patch elements where they pad K less than blocks of 128 (K = 576: 3 blocks instead of 5)
            const int pad2 = (g.K + 127) / 128 * 128 - g.K, pad3 = (g.K + 191) / 192 * 192 - g.K;
            if (pad3 < pad2) return launch_fast_pf<3, 4, 2>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
            return launch_fast_pf<2, 4, 2>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
        }
        if (g.F % 16 == 0) { *done = true; return launch_fast_pf<2, 4, 1>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s); }
    }
    if ((g.B & 3) == 0 && va == 2) {
        if (g.F % 64 == 0) { *done = true; return launch_fast_pf<2, 2, 4>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s); }
        if (g.F % 32 == 0) { *done = true; return launch_fast_pf<4, 2, 2>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s); }
        if (g.F % 16 == 0) { *done = true; return launch_fast_pf<4, 2, 1>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s); }
    }
    return LC_OK;
}

}  // namespace

namespace {

// the masked kernel (any shape), filter tiles per wave by F
template <typename T>
int launch_backward_weights_generic(const Geom &g, const T *x1, const T *dy1, const T *x2, const T *dy2, float beta,
                                    float gamma, float *out, float *ssq, int *kblocks_out, hipStream_t s) {
    if (g.F <= 16) return launch_nt<1>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
    if (g.F <= 32) return launch_nt<2>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
    return launch_nt<4>(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
}

}  // namespace

int launch_backward_weights_f32(const Geom &g, const float *x1, const float *dy1, const float *x2, const float *dy2,
                                float beta, float gamma, float *out, hipStream_t s, float *ssq, int *kblocks_out) {
    {
        bool done = false;
        const int rc = launch_backward_weights_fast_path(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s, &done);
        if (done) return rc;
    }
    return launch_backward_weights_generic(g, x1, dy1, x2, dy2, beta, gamma, out, ssq, kblocks_out, s);
}

int launch_backward_weights_bf16_storage(const Geom &g, const void *x, const void *dy, float beta, float *dw,
                                         hipStream_t s) {
    const bf16_t *none = nullptr;
    bool done = false;
    const int rc = launch_backward_weights_fast_path(g, (const bf16_t *)x, (const bf16_t *)dy, none, none, beta, 1.f, dw,
                                                     nullptr, nullptr, s, &done);
    if (done) return rc;
    return launch_backward_weights_generic(g, (const bf16_t *)x, (const bf16_t *)dy, none, none, beta, 1.f, dw, nullptr,
                                           nullptr, s);
}

}  // namespace lc
