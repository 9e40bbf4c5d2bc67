/*
 * rmsnorm.h -- C ABI of the fused RMS layer norm of the MI355X (gfx950) library.
 *
 * The paper's second kernel (section "Method and Investigated Kernels": the RMS layernorm, "typically
 * the second most computationally expensive" kernel of an LLM; Table I lists it fused, as in the
 * serving stack it is compared with; Fig. 3 shows its results).  The operation is Zhang and
 * Sennrich's root-mean-square layer normalisation with an optional residual add in front:
 *
 *     z[t, :]     = x[t, :] + residual[t, :]            (z = x when residual == NULL)
 *     out[t, i]   = z[t, i] / sqrt(mean_i z[t, i]^2 + eps) * weight[i]
 *     residual[t] = z[t]                                 (written back in place)
 *
 * The sum z, its mean square and the product are taken in fp32 from the bf16 (or fp16) inputs; out
 * and the new residual are rounded to the element type (nearest even) once.  One pass over HBM: every row is read once and
 * written once, held in registers in between.
 *
 * Conventions are those of attn.h: every pointer in rmsnorm_args is a DEVICE pointer owned by the
 * caller, strides are in ELEMENTS, the hidden dimension is contiguous, rows and `weight` are 16-byte
 * aligned.  rmsnorm_fused_add only validates host-visible fields, picks a kernel instance and
 * enqueues one kernel on `hip_stream`; it never allocates, synchronises or copies, and may be captured
 * in a HIP graph.  Errors visible to the host come back as a negative attn_status (see attn.h) and
 * nothing is enqueued.  `out` may alias `x`; `residual` must not overlap `x` or `out`.
 */
#ifndef RMSNORM_H_
#define RMSNORM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rmsnorm_args {
    uint32_t struct_bytes; /* = sizeof(rmsnorm_args) */
    int32_t dtype;         /* ATTN_BF16 (1) or ATTN_F16 (2) for x, residual, weight and out; else ATTN_ERR_DTYPE */
    int32_t num_tokens;    /* T rows; 0 is allowed (nothing happens) */
    int32_t hidden;        /* H, a multiple of 8, at most 16384 */
    const void *x;         /* [T, H] */
    int64_t x_stride;      /* elements between rows, a multiple of 8 */
    void *residual;        /* NULL, or [T, H] read and overwritten with x + residual */
    int64_t residual_stride;
    const void *weight; /* [H] */
    void *out;          /* [T, H] */
    int64_t out_stride;
    float eps; /* added to the mean square */
} rmsnorm_args;

/* Enqueues the fused (residual add +) RMS norm.  Returns ATTN_OK or a negative attn_status. */
int rmsnorm_fused_add(const rmsnorm_args *args, void *hip_stream);

/* Ahead-of-time tuning for the shape bucket of `shape_like` (hidden size, residual or not, token
 * count rounded up to a power of two): times every valid compiled instance on synthetic buffers that
 * the call allocates and frees, then times the three fastest and the built-in choice again taking
 * turns launch by launch, keeps the fastest of those (the built-in choice keeps ties within 3 %) and,
 * if cache_path is not NULL, merges it into the same cache file attn_tune uses.  `iters` timed
 * launches per instance and pass (<= 0: a default).
 * Synchronous; not capturable.  flags: bit 0 = one line per instance on stderr. */
int rmsnorm_tune(const rmsnorm_args *shape_like, const char *cache_path, int iters, int flags);

/* Introspection (pure host functions), as for attention. */
int rmsnorm_num_instances(void);
int rmsnorm_instance_name(int id, char *buf, size_t buf_bytes);
int rmsnorm_selected_instance(const rmsnorm_args *args);
void rmsnorm_force_instance(int id); /* -1 = automatic */

#ifdef __cplusplus
}
#endif
#endif /* RMSNORM_H_ */
