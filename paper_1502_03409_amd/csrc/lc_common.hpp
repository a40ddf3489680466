// Shared host/device helpers of the HIP path: derived geometry, MFMA wrappers, launch bookkeeping.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <initializer_list>

#include "../../include/lc.h"
#include "../../include/lc_plan.h"

namespace lc {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Layer geometry with the derived sizes (Sec. 3.1: valid fields of size R at stride S).
struct Geom {
    int B, H, W, C, R, S, F;
    int LH, LW, L, K, RC;  // RC = R*C: one patch row, contiguous in an [H][W][C] image
};

inline bool make_geom(const lc_geom_t *g, Geom *o) {
    if (!g) return false;
    if (g->B < 1 || g->H < 1 || g->W < 1 || g->C < 1 || g->R < 1 || g->S < 1 || g->F < 1) return false;
    if (g->R > g->H || g->R > g->W) return false;
    o->B = g->B; o->H = g->H; o->W = g->W; o->C = g->C; o->R = g->R; o->S = g->S; o->F = g->F;
    o->LH = (g->H - g->R) / g->S + 1;
    o->LW = (g->W - g->R) / g->S + 1;
    o->L = o->LH * o->LW;
    const long long K = (long long)g->R * g->R * g->C;
    if (K > (1 << 24)) return false;
    o->K = (int)K;
    o->RC = g->R * g->C;
    // element counts must stay inside 31-bit indices (the kernels index with 32-bit offsets per image / location
    // and 64-bit bases)
    const long long img = (long long)g->H * g->W * g->C;
    const long long wl = K * g->F;
    if (img > (1LL << 30) || wl > (1LL << 30) || (long long)o->L * g->F > (1LL << 30)) return false;
    return true;
}

// MI355X: 256 compute units in 8 XCDs; consecutive workgroup ids go to consecutive XCDs.
// remap_xcd turns a hardware workgroup id into a work index such that each XCD walks a
// contiguous range of work (neighbouring work items share image rows and thus L2 lines).
constexpr int kXcds = 8;
__device__ __forceinline__ int remap_xcd(int wg, int n_wg) {
    const int per = (n_wg + kXcds - 1) / kXcds;
    const int full = n_wg - (per - 1) * kXcds;  // number of XCDs that get `per` items (1..8)
    const int xcd = wg % kXcds, slot = wg / kXcds;
    // XCDs [0,full) own `per` items each, the rest own per-1
    const int start = xcd < full ? xcd * per : full * per + (xcd - full) * (per - 1);
    return start + slot;
}

// v_mfma_f32_16x16x4_f32: D[16x16] += A[16x4] * B[4x16].
// Lane l supplies A[l%16][l/16] and B[l/16][l%16]; it receives D[4*(l/16)+r][l%16] in component r.
__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// N consecutive fp32 values as one vector register group
template <int N> struct FVec;
template <> struct FVec<1> { typedef float T; };
template <> struct FVec<2> { typedef float T __attribute__((ext_vector_type(2))); };
template <> struct FVec<4> { typedef float T __attribute__((ext_vector_type(4))); };
template <int N>
__device__ __forceinline__ float fget(const typename FVec<N>::T &v, int i) {
    if constexpr (N == 1) return v; else return v[i];
}


// ---------------------------------------------------------------------------------------------
// Loads whose waits are written by hand.  The kernels that use them keep a fixed program order of their memory
// operations and wait with explicit counts (the memory counter retires loads, and on this chip stores, in the order
// they were issued), because the compiler's wait insertion, which does not know the order of a loop's iterations,
// waits for more than is needed and so for loads that have just been issued.  Inline assembly is invisible to that
// insertion: nothing here is waited for unless the kernel says so.
typedef const __attribute__((address_space(1))) char *gbyte_ptr;

// The base pointers and LDS addresses below are "s" operands: a value the compiler does not hold in scalar registers
// fails to assemble (it is never moved there silently).  Every memory instruction is preceded by five wait states
// (s_nop 4): that is what the hardware needs between a vector-ALU write of a scalar register (a v_readfirstlane the
// compiler may have scheduled right in front of the statement) and a memory instruction that reads it as its base,
// and the compiler's hazard handling does not look inside inline assembly.  It also covers the one wait state between
// the write of m0 and the LDS-direct load that uses it.
//
// 16 bytes per lane from base + off straight into LDS: lane i's vector lands at lds_addr + 16 i (lds_addr: byte
// address inside the workgroup's LDS, the same for the whole wave, as is base)
__device__ __forceinline__ void load_lds16(gbyte_ptr base, unsigned off, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(off), "s"(base)
                 : "memory");
}
// N consecutive floats (1, 2 or 4) per lane from base + off into registers; the value may be used only after
// wait_loads has been called on it
template <int N>
__device__ __forceinline__ typename FVec<N>::T load_nowait(gbyte_ptr base, unsigned off) {
    typename FVec<N>::T v;
    if constexpr (N == 1)
        asm volatile("s_nop 4\n\tglobal_load_dword %0, %1, %2" : "=&v"(v) : "v"(off), "s"(base) : "memory");
    else if constexpr (N == 2)
        asm volatile("s_nop 4\n\tglobal_load_dwordx2 %0, %1, %2" : "=&v"(v) : "v"(off), "s"(base) : "memory");
    else
        asm volatile("s_nop 4\n\tglobal_load_dwordx4 %0, %1, %2" : "=&v"(v) : "v"(off), "s"(base) : "memory");
    return v;
}
// one float per lane to base + off; counted by the memory counter like a load, never waited for unless the kernel does
__device__ __forceinline__ void store_nowait(gbyte_ptr base, unsigned off, float v) {
    asm volatile("s_nop 4\n\tglobal_store_dword %0, %1, %2" ::"v"(off), "v"(v), "s"(base) : "memory");
}
// wait until at most N of the memory operations issued so far are in flight; v: a value one of the finished loads
// delivers (ties the wait to the value's uses)
template <int N, typename V>
__device__ __forceinline__ void wait_loads(V &v) {
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(v) : "n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// wait_loads<BASE - d>(v) for a d in 0..MAXD that is a constant only after the surrounding loop has been unrolled
template <int BASE, int MAXD, typename V>
__device__ __forceinline__ void wait_loads_minus(int d, V &v) {
    if constexpr (MAXD == 0) {
        wait_loads<BASE>(v);
    } else {
        if (d == MAXD) wait_loads<BASE - MAXD>(v);
        else wait_loads_minus<BASE, MAXD - 1>(d, v);
    }
}

// Operand storage.  T = float, or bf16_t: bf16 bit patterns that are widened to fp32 (exactly) on their way to
// LDS or to the B operand, so the same fp32 MFMAs serve both; bf16 storage halves the bytes fetched.
typedef unsigned short bf16_t;
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
template <typename T, int N> struct RawVec { typedef typename FVec<N>::T V; };            // N consecutive elements as loaded
template <> struct RawVec<bf16_t, 1> { typedef unsigned short V; };
template <> struct RawVec<bf16_t, 2> { typedef unsigned int V; };
template <> struct RawVec<bf16_t, 4> { typedef u32x2 V; };
__device__ __forceinline__ float bf16_lo(unsigned int v) { return __builtin_bit_cast(float, v << 16); }
__device__ __forceinline__ float bf16_hi(unsigned int v) { return __builtin_bit_cast(float, v & 0xffff0000u); }
// element i of a raw vector of N, as fp32
template <typename T, int N>
__device__ __forceinline__ float raw_get(const typename RawVec<T, N>::V &v, int i) {
    if constexpr (sizeof(T) == 4) {
        return fget<N>(v, i);
    } else if constexpr (N == 1) {
        return bf16_lo(v);
    } else if constexpr (N == 2) {
        return (i & 1) ? bf16_hi(v) : bf16_lo(v);
    } else {
        return (i & 1) ? bf16_hi(v[i >> 1]) : bf16_lo(v[i >> 1]);
    }
}
// one stored element as fp32
template <typename T>
__device__ __forceinline__ float ld_f32(const T *p) {
    if constexpr (sizeof(T) == 4) return *p;
    else return bf16_lo(*p);
}
template <typename T>
__device__ __forceinline__ f32x4 raw_widen4(const typename RawVec<T, 4>::V &v) {
    if constexpr (sizeof(T) == 4) return v;
    else return (f32x4){bf16_lo(v[0]), bf16_hi(v[0]), bf16_lo(v[1]), bf16_hi(v[1])};
}

// v_mfma_f32_16x16x16_bf16: D[16x16] += A[16x16] * B[16x16] with bf16 operands.  Lane l supplies the four
// consecutive contraction indices 4*(l/16) .. +3 of row (A) or column (B) l%16, packed two per register; D as above.
typedef short bf16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4 mfma16_bf16(u32x2 a, u32x2 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(bf16x4, a), __builtin_bit_cast(bf16x4, b), c,
                                                     0, 0, 0);
}

// A store whose line nobody reads again soon (a weight gradient far larger than the caches, written once): marked
// non-temporal, so that it does not push the kernel's operands out of the L2 and the Infinity Cache on its way out.
template <typename V>
__device__ __forceinline__ void stream_store(const V &v, V *p) {
    __builtin_nontemporal_store(v, p);
}

void set_hip_error(hipError_t e, const char *where);
void set_error_text(const char *text);

// ---------------------------------------------------------------------------------------------
// Launch plans.  A launcher writes the launch down first (LaunchPlan), runs the host check that belongs to
// the kernel family (check_* next to each kernel: the tiles cover the problem exactly once, a chunk fits the
// staging registers and the LDS, clamped addresses stay inside the tensors) and then goes through LC_LAUNCH,
// which applies the limits every launch has, and either launches or, inside lc_plan_query, keeps the record.
typedef lc_launch_t LaunchPlan;

LaunchPlan make_plan(const char *kernel, std::initializer_list<int> tparam, std::initializer_list<int> arg, dim3 grid,
                     unsigned block, size_t lds_bytes);
// grid, block and LDS limits of the device; LC_OK or LC_EINTERNAL
int check_launch_shape(const LaunchPlan &p);
// records "<kernel>: <what>" as the thread's last error and returns LC_EINTERNAL
int plan_fail(const LaunchPlan &p, const char *what);
bool plan_capture();                          // true on a thread that is inside lc_plan_query
void plan_capture_add(const LaunchPlan &p);

#define LC_PLAN_REQUIRE(p, cond)                                  \
    do {                                                          \
        if (!(cond)) return lc::plan_fail(p, #cond);              \
    } while (0)

// Launch `kern` as planned in `plan` (or only record the plan).  `where` names the launch in error messages.
#define LC_LAUNCH(plan, where, kern, stream, ...)                                                              \
    do {                                                                                                       \
        if (int rc_shape__ = lc::check_launch_shape(plan)) return rc_shape__;                                  \
        if (lc::plan_capture()) {                                                                              \
            lc::plan_capture_add(plan);                                                                        \
            break;                                                                                             \
        }                                                                                                      \
        if (int rc_lds__ = lc::allow_dynamic_lds((const void *)(kern), (size_t)(plan).lds_bytes, where))       \
            return rc_lds__;                                                                                   \
        hipLaunchKernelGGL(kern, dim3((plan).grid[0], (plan).grid[1], (plan).grid[2]), dim3((plan).block),     \
                           (size_t)(plan).lds_bytes, stream, __VA_ARGS__);                                     \
        LC_HIP_LAUNCH_CHECK(where);                                                                            \
    } while (0)

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// argument checks shared by the entry points that take a [B,H,W,C] map
inline int check_map_dims(int32_t B, int32_t H, int32_t W, int32_t C) {
    if (B < 1 || H < 1 || W < 1 || C < 1) return LC_EINVAL;
    if ((long long)H * W * C > (1LL << 30) || (long long)B * H * W > (1LL << 40)) return LC_EINVAL;
    return LC_OK;
}
inline bool ptr_aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }
// everything lcn_variant_bwd checks before it looks at its workspace
inline int check_lcn_variant_bwd_args(const float *x, const float *mu, const float *rstd, const float *dy, float *dx,
                                      int32_t B, int32_t H, int32_t W, int32_t C, int32_t ksize, float gauss_sigma,
                                      uint32_t flags) {
    if (check_map_dims(B, H, W, C) != LC_OK || (flags & ~7u)) return LC_EINVAL;
    if (ksize < 1 || ksize > 15 || (ksize & 1) == 0 || !(gauss_sigma > 0.f)) return LC_EINVAL;
    if (!x || !mu || !rstd || !dy || !dx) return LC_ENULL;
    if (!ptr_aligned16(x) || !ptr_aligned16(mu) || !ptr_aligned16(rstd) || !ptr_aligned16(dy) || !ptr_aligned16(dx))
        return LC_EALIGN;
    if (dx == x || dx == dy) return LC_EINVAL;
    return LC_OK;
}

// raises a kernel's dynamic LDS limit when `bytes` needs it (once per kernel and device); LC_OK or LC_EHIP
int allow_dynamic_lds(const void *kernel, size_t bytes, const char *where);

#define LC_HIP_LAUNCH_CHECK(where)                       \
    do {                                                 \
        hipError_t e__ = hipGetLastError();              \
        if (e__ != hipSuccess) {                         \
            lc::set_hip_error(e__, where);               \
            return LC_EHIP;                              \
        }                                                \
    } while (0)

// Batch tile of the workgroup-tiled kernels in units of 32 images: 4, 3 (if allowed) or 2, whichever pads the
// batch least; the larger tile on a tie.
inline int batch_tile_mt(int B, bool allow3) {
    int best = 4, waste = 1 << 30;
    for (int mt = 4; mt >= 2; --mt) {
        if (mt == 3 && !allow3) continue;
        const int bt = 32 * mt, wst = (B + bt - 1) / bt * bt - B;
        if (wst < waste) { waste = wst; best = mt; }
    }
    return best;
}

// kernels' host launchers (one per translation unit)
// alpha_dev (nullable): device scalar that overrides alpha
int launch_forward_f32(const Geom &g, const float *x, const float *w, const float *bias, float alpha,
                       const float *alpha_dev, float *y, hipStream_t s, void *ws = nullptr, size_t ws_bytes = 0);
int launch_l2pool_fwd(const float *x, float *y, int B, int H, int W, int C, int ks, int st, float eps, hipStream_t s);
int launch_l2pool_bwd(const float *x, const float *y, const float *dy, float *dx, int B, int H, int W, int C, int ks,
                      int st, hipStream_t s);
// Statistics pooled over the channels.  mode 0: forward (out = y; mu, rstd written).  mode 1: backward (out = dx;
// mu, rstd read).  modes 2..5: the passes of the two-stage form (mean; divide; gradient up to dv and the field of
// its channel sums; dx = dv - window sum of field), field = B*H*W floats of scratch for modes 4 and 5.
// zero_pad: pixels outside the image count as zeros and the window keeps its full-window normalisation.
int launch_lcn(int mode, const float *x, const float *dy, float *out, float *mu, float *rstd, int B, int H, int W,
               int C, int ks, float sigma, float eps, hipStream_t s, int zero_pad = 0, float *field = nullptr);
// 3x3 stride-1 pooling and the one-stage pooled LCN of its result in one kernel; *done: whether the shape took it
int launch_pool_lcn_fused(const float *x, float *p, float *out, float *mu, float *rstd, int B, int H, int W, int C,
                          float peps, int ks, float sigma, float eps, hipStream_t s, bool *done);
// lcn_bwd followed by l2pool_bwd (the gradient of pooling + LCN with respect to the pooling input)
int launch_lcn_pool_bwd(const float *x, const float *p, const float *mu, const float *rstd, const float *dn,
                        float *scratch, float *dx, int B, int H, int W, int C, int pks, int pst, int ks, float sigma,
                        hipStream_t s);
// LCN variants (flags as in lc.h: per-channel statistics, zero-padded borders, two stages)
size_t lcn_variant_scratch_bytes(int B, int H, int W, int C, unsigned flags);
int launch_lcn_variant_fwd(const float *x, float *y, float *mu, float *rstd, int B, int H, int W, int C, int ks,
                           float sigma, float eps, unsigned flags, hipStream_t s);
int launch_lcn_variant_bwd(const float *x, const float *mu, const float *rstd, const float *dy, float *dx, int B, int H,
                           int W, int C, int ks, float sigma, unsigned flags, void *ws, size_t ws_bytes, hipStream_t s);
// wide layers (128-filter blocks): workgroup-tiled forward; LC_EUNSUPPORTED outside forward_wide_supported()
bool forward_wide_supported(const Geom &g);
size_t forward_wide_workspace_bytes(const Geom &g);   // optional workspace: K-slices for layers with few fields
int launch_forward_wide_f32(const Geom &g, const float *x, const float *w, const float *bias, float alpha,
                            const float *alpha_dev, float *y, void *ws, size_t ws_bytes, hipStream_t s);
// cells of 128-value blocks: workgroup-tiled backward data; LC_EUNSUPPORTED outside backward_data_wide_supported()
bool backward_data_wide_supported(const Geom &g);
bool backward_data_dense_supported(const Geom &g);   // one field covering the whole input
int launch_backward_data_wide_f32(const Geom &g, const float *dy, const float *w, float *dx, hipStream_t s);
// bf16 operands (raw 16-bit patterns), fp32 results; LC_EUNSUPPORTED for shapes outside the aligned set
int launch_forward_bf16(const Geom &g, const void *x, const void *w, const float *bias, float alpha, float *y,
                        hipStream_t s);
int launch_backward_data_bf16(const Geom &g, const void *dy, const void *w, float *dx, hipStream_t s);
// bf16 storage through the fp32 kernels' structure: the pipelined kernels for the aligned shapes (bf16 MFMAs in the
// backward-data pass, operands widened on the way in elsewhere), the masked kernels for every other shape
bool backward_data_bf16_pipelined_supported(const Geom &g);
int launch_forward_bf16_storage(const Geom &g, const void *x, const void *w, const float *bias, float alpha, float *y,
                                hipStream_t s);
int launch_backward_data_bf16_storage(const Geom &g, const void *dy, const void *w, float *dx, hipStream_t s);
int launch_backward_weights_bf16_storage(const Geom &g, const void *x, const void *dy, float beta, float *dw,
                                         hipStream_t s);
// strip-sharing bf16 forward for patch rows that are not multiples of 16 values and filters in blocks of 16 or 32
bool bf16_strip_forward_supported(const Geom &g);
int launch_forward_bf16_strip(const Geom &g, const void *x, const void *w, const float *bias, float alpha, float *y,
                              hipStream_t s);
// bf16 weight gradient for patch rows in whole 4-value vectors and filters in blocks of 16 (batches in steps of 16)
bool bf16_rows_backward_weights_supported(const Geom &g);
int launch_backward_weights_bf16_rows(const Geom &g, const void *x, const void *dy, float beta, float *dw,
                                      hipStream_t s);
// workgroup-tiled bf16 forward for wide layers; LC_EUNSUPPORTED outside bf16_tiled_forward_supported()
bool bf16_tiled_forward_supported(const Geom &g);
int launch_forward_bf16_tiled(const Geom &g, const void *x, const void *w, const float *bias, float alpha, float *y,
                              hipStream_t s);
bool bf16_tiled_backward_data_supported(const Geom &g);
int launch_backward_data_bf16_tiled(const Geom &g, const void *dy, const void *w, float *dx, hipStream_t s);
bool bf16_tiled_backward_weights_supported(const Geom &g);
int launch_backward_weights_bf16_tiled(const Geom &g, const void *x, const void *dy, float beta, float *dw,
                                       hipStream_t s);
int launch_backward_weights_bf16(const Geom &g, const void *x, const void *dy, float beta, float *dw, hipStream_t s);
size_t sae_workspace_bytes(const Geom &g);
int launch_sae_step(const Geom &g, const float *x, float *w, float *b, float *alpha, float lambda, float eps_sparse,
                    float lr, uint32_t flags, float *h_out, float *cost_out, void *ws, hipStream_t s);
int launch_backward_data_f32(const Geom &g, const float *dy, const float *w, float *dx, hipStream_t s);
// out[l,k,f] = beta*out + gamma * sum over pairs p of sum_b patch(x_p)[b,l,k] * dy_p[b,l,f]; x2/dy2 may be NULL.
// ssq (nullable): receives, per location, block of patch elements and filter, the sum of squares of the values
// stored, as [L][*kblocks_out][F] floats; at most backward_weights_max_kblocks(g) blocks per location.
int launch_backward_weights_f32(const Geom &g, const float *x1, const float *dy1, const float *x2, const float *dy2,
                                float beta, float gamma, float *out, hipStream_t s, float *ssq = nullptr,
                                int *kblocks_out = nullptr);
inline int backward_weights_max_kblocks(const Geom &g) { return (g.K + 63) / 64; }   // the smallest block is 64 rows

}  // namespace lc
