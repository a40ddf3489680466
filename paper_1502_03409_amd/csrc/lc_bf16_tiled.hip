// bf16-operand forward contraction, workgroup-tiled (Eq. 1 encoder term, Sec. 3.1 geometry).
//
// A workgroup owns one field, 128 of its filters and a batch tile of 32*MT images; its four waves form a
// 2 x 2 grid (16*MT images x 64 filters each).  The field's patch rows reach the waves through LDS in
// chunks of 64 contraction indices (128 contiguous bytes per image, two buffers, one barrier per chunk);
// the filters go straight from global memory to registers, one step of 32 indices ahead: lane (n, kk)
// loads rows 8kk..8kk+7 of the step at filters 4n..4n+3 (16 lanes cover whole 128-byte lines) and two
// 4x4 register transposes turn them into the k-contiguous operands of v_mfma_f32_16x16x32_bf16 for the
// four filter tiles, in which column n of tile u is filter 4n+u.
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

template <int MT>
__global__ __launch_bounds__(256) void lc_forward_bf16_tiled_kernel(Geom g, const unsigned short *__restrict__ x,
                                                                    const unsigned short *__restrict__ w,
                                                                    const float *__restrict__ bias, float alpha,
                                                                    float *__restrict__ y, int fblocks, int btiles) {
    constexpr int BT = 32 * MT, NS = MT;          // NS: 16-byte staging slots per thread and chunk
    constexpr int BUF = BT * kRowBytes;
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

    // staging: slot s moves 16 bytes (segment tid&7) of image (tid>>3) + 32 s; images beyond the batch
    // repeat image B-1 and their results are never stored
    const int seg = tid & 7, brow = tid >> 3;
    int xoff[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int b = min(b0 + brow + 32 * s, g.B - 1);
        xoff[s] = (b * g.H + i * g.S) * WC + j * g.S * g.C + seg * 8;
    }
    u32x4 st[NS];
    auto stage_load = [&](int c) {
        const int kh = c / cpr;
        const int o = kh * WC + (c - kh * cpr) * kChunk;
#pragma unroll
        for (int s = 0; s < NS; ++s) st[s] = *(g4_ptr)((gh_ptr)x + xoff[s] + o);
    };
    auto stage_store = [&](int buf) {
#pragma unroll
        for (int s = 0; s < NS; ++s) *(u32x4 *)(xs + buf * BUF + (brow + 32 * s) * kRowBytes + seg * 16) = st[s];
    };
    // filters: the chunks tile k contiguously, so step q covers rows 32q .. 32q+31 of the field's K x F matrix
    gh_ptr wl = (gh_ptr)w + (size_t)loc * g.K * g.F + f0 + 4 * n + (size_t)(8 * kk) * g.F;
    auto wload = [&](int q, u32x2 (&r)[8]) {
        gh_ptr p = wl + (size_t)(32 * q) * g.F;
#pragma unroll
        for (int t = 0; t < 8; ++t) r[t] = *(g2_ptr)(p + t * g.F);
    };

    u32x2 wr0[8], wr1[8];
    stage_load(0);
    wload(0, wr0);
    wload(1, wr1);
    stage_store(0);
    if (nchunks > 1) stage_load(1);
    __syncthreads();
    const int arow = (wm * 16 * MT + n) * kRowBytes + 16 * kk;
    for (int c = 0; c < nchunks; ++c) {
        const unsigned char *ab = xs + (c & 1) * BUF + arow;
        u32x4 bo[4];
        transpose8x4_bf16(wr0, bo);
        wload(min(2 * c + 2, nsteps - 1), wr0);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const u32x4 a = *(const u32x4 *)(ab + mt * 16 * kRowBytes);
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[mt][u] = mfma32_bf16(a, bo[u], acc[mt][u]);
        }
        transpose8x4_bf16(wr1, bo);
        wload(min(2 * c + 3, nsteps - 1), wr1);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const u32x4 a = *(const u32x4 *)(ab + mt * 16 * kRowBytes + 64);
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[mt][u] = mfma32_bf16(a, bo[u], acc[mt][u]);
        }
        // the other buffer was last read in chunk c-1, which every wave left at the previous barrier
        if (c + 1 < nchunks) {
            stage_store((c + 1) & 1);
            if (c + 2 < nchunks) stage_load(c + 2);
        }
        __syncthreads();
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

template <int MT>
int launch_tiled(const Geom &g, const void *x, const void *w, const float *bias, float alpha, float *y,
                 hipStream_t s) {
    constexpr int BT = 32 * MT;
    const size_t lds = (size_t)2 * BT * kRowBytes;
    auto kern = lc_forward_bf16_tiled_kernel<MT>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { set_hip_error(e, "lc_forward (bf16): hipFuncSetAttribute"); return LC_EHIP; }
    }
    const int fblocks = g.F / 128, btiles = (g.B + BT - 1) / BT;
    hipLaunchKernelGGL(kern, dim3((unsigned)(g.L * fblocks * btiles)), dim3(256), lds, s, g,
                       (const unsigned short *)x, (const unsigned short *)w, bias, alpha, y, fblocks, btiles);
    LC_HIP_LAUNCH_CHECK("lc_forward (bf16, tiled) launch");
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
#ifndef LC_TILED_FORCE_MT4
    if (g.B > 128) return launch_tiled<8>(g, x, w, bias, alpha, y, s);
#endif
    return launch_tiled<4>(g, x, w, bias, alpha, y, s);
}

}  // namespace lc
