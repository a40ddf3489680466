/*
 * lc_plan.h - host-only introspection of the launch plans behind lc.h's layer primitives.
 *
 * Every launcher of the library first writes down the launch it is about to make (kernel family,
 * compile-time tile parameters, the scalars that fix the kernel's indexing, grid, block and LDS bytes),
 * checks that record on the host against what the kernel assumes (tiles cover the problem exactly,
 * staging registers and LDS hold a chunk, clamped addresses stay inside the tensors) and only then
 * launches.  lc_plan_query runs the same planning and the same checks for a geometry without touching
 * the GPU and hands back the records, so that tests and tools can walk many geometries on a machine
 * that has no GPU at all.  A plan that fails its checks is a bug in the library: the call returns
 * LC_EINTERNAL, lc_last_error() names the violated condition, and nothing is launched.
 */
#ifndef LC_PLAN_H_
#define LC_PLAN_H_

#include "lc.h"

#ifdef __cplusplus
extern "C" {
#endif

/* One planned kernel launch.  `kernel` names the kernel family; the meaning of tparam[] (compile-time
 * parameters of the chosen instance) and arg[] (runtime scalars) is per family and listed next to each
 * kernel's host check in the sources; unused entries are zero. */
typedef struct {
    char kernel[32];
    int32_t tparam[12];
    int32_t arg[12];
    uint32_t grid[3];
    uint32_t block;
    uint64_t lds_bytes;
} lc_launch_t;

/* Host only.  Plans `op` (an lc_op: the three layer primitives of Sec. 3.1 / Eq. 1, or LC_OP_SAE_STEP for
 * the whole training step) for geometry g and operand dtype exactly as the entry point would, with every
 * host check applied, and writes up to max_out records to out (out may be NULL if max_out is 0).  *n_out
 * receives the number of launches planned, which may exceed max_out.  LC_OP_FORWARD is planned with its
 * optional workspace present.  Returns LC_OK, LC_EINVAL (geometry, op or dtype), LC_EUNSUPPORTED (no kernel
 * for this shape and dtype) or LC_EINTERNAL. */
int lc_plan_query(const lc_geom_t *g, int op, int dtype, lc_launch_t *out, int32_t max_out, int32_t *n_out);

/* Host only.  The launch l2pool_lcn_fwd would make for a [B,H,W,C] map where it runs as one kernel, planned and
 * checked as in the call: *n_out = 1 and out[0] holds it; *n_out = 0 where the call runs l2pool_fwd's and lcn_fwd's
 * kernels one after the other (those keep no plan records).  Returns LC_OK, LC_EINVAL or LC_EINTERNAL. */
int l2pool_lcn_plan_query(int32_t B, int32_t H, int32_t W, int32_t C, int32_t pool_ksize, int32_t pool_stride,
                          int32_t lcn_ksize, float gauss_sigma, lc_launch_t *out, int32_t max_out, int32_t *n_out);

#ifdef __cplusplus
}
#endif
#endif /* LC_PLAN_H_ */
