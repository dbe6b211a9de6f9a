/*
 * libfq -- fused learnable-scale fake quantization for AMD MI355X (gfx950).
 *
 * C ABI.  Every tensor pointer in fq_tensor is a DEVICE pointer owned by the
 * caller; descriptor structs and arrays of them are HOST memory.  The library
 * enqueues kernels on the given HIP stream and returns; it never synchronises
 * the device and never allocates or frees device memory.  (The three calls that
 * copy a descriptor table to the device -- fq_multi_tensor, fq_plan_create,
 * fq_plan_run_adam -- stage it in pinned HOST memory; see fq_multi_tensor for
 * what that implies.)  All functions return
 * an fq_status (0 = success, negative = failure); validation happens before
 * anything is enqueued, so a failing call has no device side effects.  Nothing
 * throws or aborts across this boundary.
 *
 * The operation (DPVO-QAT++, Sec. 3.2):
 *   scale     s_c = clip(softplus(theta_c) + eps, s_min, s_max)        Eq. (3)-(4)
 *   forward   y   = s_c * round(clip(x / s_c, qmin, qmax))             Eq. (5)-(6)
 *   backward  straight-through estimator (round differentiated as identity):
 *             gx = gy where qmin <= x/s_c <= qmax, else +0
 *             gs_c = sum over the channel of gy * t,
 *                    t = round(x/s_c) - x/s_c inside the range, qmin below, qmax above
 *             gtheta_c = gs_c * sigmoid(theta_c), or 0 where the clip of Eq. (3)-(4) is active
 * round() is round-half-to-even; x/s is the correctly rounded binary32 quotient;
 * all arithmetic is binary32 (softplus/sigmoid evaluated in binary64 and rounded
 * once); FP16 tensors are widened exactly and narrowed with round-to-nearest-even
 * (Sec. 3.3 "Mixed precision").  Results are bitwise reproducible run to run.
 *
 * Layout: every tensor is a contiguous [outer, channels, inner] array; element
 * (o, c, k) uses scale c.
 *   per-channel NCHW activation:        outer = N, channels = C,     inner = H*W
 *   per-output-channel conv weight:     outer = 1, channels = C_out, inner = C_in*kh*kw
 *   per-tensor (the paper's activations): outer = 1, channels = 1,   inner = numel
 */
#ifndef FQ_H
#define FQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum fq_status {
    FQ_OK = 0,
    FQ_ERR_NULL = -1,          /* a required pointer is NULL */
    FQ_ERR_DTYPE = -2,         /* dtype is not FQ_F16 / FQ_F32 */
    FQ_ERR_SHAPE = -3,         /* negative extent, element/slab/block count overflow, bad n or mode */
    FQ_ERR_QRANGE = -4,        /* need qmin <= 0 <= qmax, qmin < qmax, |q| <= 32768; int8 codes need [-128,127] */
    FQ_ERR_ALIGN = -5,         /* pointer not aligned to its element size (workspace: 256 bytes) */
    FQ_ERR_WORKSPACE = -6,     /* workspace NULL or smaller than fq_workspace_bytes() */
    FQ_ERR_SCALE_PARAMS = -7,  /* need finite eps, 0 < s_min <= s_max, no NaN */
    FQ_ERR_LAUNCH = -8,        /* the HIP runtime reported an error while enqueuing */
    FQ_ERR_ALIAS = -9,         /* output partially overlaps its input (exact in-place is allowed; q may not
                                  overlap x or y at all) */
    FQ_ERR_OPTIMIZER = -10     /* bad fq_adam: step < 1, beta outside [0,1), lr/eps not finite or eps < 0 */
} fq_status;

typedef enum fq_dtype { FQ_F16 = 0, FQ_F32 = 1 } fq_dtype;

enum {
    /* Backward: do not write gx.  For tensors whose values are frozen and only the
       scales train (the paper's weights, Sec. 3.2 "Scale-Only QAT"). */
    FQ_FLAG_NO_DX = 1u,
    /* Backward: finish the per-channel scale gradient in a second small kernel instead
       of in the last block of each channel.  Same results bit for bit. */
    FQ_FLAG_TWO_PASS = 2u
};

enum { FQ_MODE_FORWARD = 1, FQ_MODE_BACKWARD = 2 };

/*
 * Optional: one Adam step on theta, fused into the end of the backward pass (the paper trains
 * only the scale parameters, with Adam: Sec. 3.2 "Training details"; it prints no
 * hyper-parameters, so they are fields).  Kingma & Ba (2015), Algorithm 1, in binary32:
 *   m <- beta1*m + (1-beta1)*g;  v <- beta2*v + ((1-beta2)*g)*g;
 *   theta_out <- theta - (lr*(m/(1-beta1^step))) / (sqrt(v/(1-beta2^step)) + eps),   g = gtheta.
 * The constants are evaluated in binary64 on the host and rounded to binary32 once each.  A
 * channel whose gradient is not finite keeps m, v and theta (the "isfinite guard" of Sec. 4.1.5).
 * Host struct; m, v, theta_out are device pointers to [channels] floats owned by the caller.
 * theta_out may be the tensor's theta itself (in place) or another buffer.
 */
typedef struct fq_adam {
    double lr, beta1, beta2, eps;     /* lr finite, 0 <= beta < 1, eps >= 0 */
    int64_t step;                     /* t >= 1: this is the t-th update */
    float *m, *v;                     /* in/out: first and second moment estimates */
    float *theta_out;                 /* out: updated parameters */
} fq_adam;

/* One tensor to fake-quantize.  Host struct; the pointers inside are device pointers. */
typedef struct fq_tensor {
    int64_t outer, channels, inner;   /* contiguous [outer, channels, inner]; any extent may be 0 */
    int32_t dtype;                    /* fq_dtype of x, y, gy, gx */
    int32_t qmin, qmax;               /* integer code range; paper: -127..127 (Eq. (5)-(6)) */
    float eps, s_min, s_max;          /* Eq. (3)-(4); plain softplus: eps = 0, s_min = FLT_MIN, s_max = +inf */
    uint32_t flags;                   /* FQ_FLAG_* */
    const void *x;                    /* in  (forward and backward) */
    void *y;                          /* out (forward); may be exactly x (in place); may be NULL if q is given */
    int8_t *q;                        /* out (forward), optional: integer codes (packed int8, one byte per
                                         element, same [outer, channels, inner] order), 0 where x is NaN */
    const float *theta;               /* in  [channels], the learnable parameter ("log scale") */
    float *s;                         /* out [channels], optional: the scales used (forward and backward) */
    const void *gy;                   /* in  (backward): upstream gradient, same dtype/shape as x */
    void *gx;                         /* out (backward); may be exactly gy; unused with FQ_FLAG_NO_DX */
    float *gs;                        /* out [channels], optional: dL/ds (overwritten) */
    float *gtheta;                    /* out [channels], optional: dL/dtheta (overwritten) */
    const fq_adam *adam;              /* host pointer, optional (backward): fused Adam step on theta */
} fq_tensor;

/*
 * Bytes of device workspace that fq_backward / fq_multi_tensor need for these n tensors
 * in this mode (a multiple of 256; at least 256).  Pure host function, touches no GPU.
 * Returns 0 if the descriptors do not validate.
 */
size_t fq_workspace_bytes(const fq_tensor *ts, int n, int mode);

/*
 * Check n descriptors for the given mode exactly as the launching calls do (everything
 * except the workspace).  Pure host function, touches no GPU.
 */
fq_status fq_validate(const fq_tensor *ts, int n, int mode);

/*
 * How the library cuts one tensor up (pure host function, touches no GPU; for tests and tuning).
 * A unit is what one partial sum of the backward covers: a block's chunk, or, for tensors whose
 * slabs are short, a whole slab handled by one wavefront (only in launches with thousands of blocks;
 * this call describes the tensor launched on its own).
 */
typedef struct fq_layout_info {
    int64_t blocks;              /* grid blocks of the forward / backward kernel */
    int64_t units_per_channel;   /* partial sums combined per channel: 1 direct, 2 exchange, 3-4 exchange
                                    tree, more: tickets (two-level when extra_slots >= 16) */
    int64_t unit_elems;          /* elements per unit (the last unit of a slab may be shorter) */
    int32_t wave_units;          /* 1: one wavefront per slab, four slabs to a block */
    int32_t extra_slots;         /* 64-bit workspace slots per channel beside the channel's own */
} fq_layout_info;
fq_status fq_layout(const fq_tensor *t, fq_layout_info *info);

/*
 * Zero a workspace on `stream` (a fill kernel, not a memset, so it may be captured in a
 * HIP graph).  A workspace must be zeroed once before its first use by fq_backward /
 * fq_multi_tensor in backward mode (memory that is already all zero, e.g. torch.zeros,
 * qualifies).  The kernels rely on it: a ticket or exchange slot that is not zero reads as a
 * unit that has already arrived, and the gradients of that channel come out wrong or are never
 * written (no kernel waits on a slot, so never a hang).  Every completed call leaves the slots
 * zero again, so the same tensor list (same shapes and flags, any pointers) may follow without
 * zeroing.  The partial sums and, for fq_multi_tensor and fq_plan_create, the descriptor table
 * stay where they were written, and where the slots lie depends on the list: before a workspace
 * serves a list of other shapes, zero it again.  One workspace must not be used by two calls
 * that can overlap in time.
 */
fq_status fq_workspace_init(void *workspace, size_t ws_bytes, void *hip_stream);

/*
 * Forward, Eq. (3)-(5), one launch: reads x, theta; writes y and, if non-NULL, q and s.
 * With y = NULL and q != NULL only the integer codes are written (1 byte per element instead
 * of 2 or 4): together with s they are the true-INT8 form of the tensor that the paper names as
 * the deployment target (Sec. 3.1, 5.2).  A tensor with zero elements is a no-op (s is still
 * written).
 */
fq_status fq_forward(const fq_tensor *t, void *hip_stream);

/*
 * STE backward for one tensor: reads x, gy, theta; writes gx (unless FQ_FLAG_NO_DX) and,
 * if non-NULL, gs, gtheta, s.  x is re-read and the quotient recomputed, nothing is saved
 * by the forward.  One launch (two with FQ_FLAG_TWO_PASS).  No float atomics: per-block
 * partial sums go to the workspace and are added in a fixed order.
 */
fq_status fq_backward(const fq_tensor *t, void *workspace, size_t ws_bytes, void *hip_stream);

/*
 * fq_backward for callers that cannot allocate device memory or may not have anyone allocate on
 * their behalf: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same inputs, outputs, flags and results (bit for bit) as fq_backward, but the
 * partial sums and slots live in a scratch array built into the library instead of a caller's
 * workspace: FQ_STATIC_SCRATCH_BYTES of device memory per GPU, held from the moment the library's
 * code is loaded on that GPU until the process ends.  The call itself allocates and frees
 * nothing, on the device or on the host, and does not synchronise.  Limits: at most
 * FQ_STATIC_MAX_UNITS partial sums (fq_layout: units_per_channel * channels) and
 * FQ_STATIC_MAX_SLOTS slots (channels * (1 + extra_slots)); a larger tensor is refused with
 * FQ_ERR_WORKSPACE before anything is enqueued.  The first call on a GPU looks the array's device
 * address up and zeroes its slots with a small fill kernel on `hip_stream`; make that call
 * outside any graph capture.  All calls on one GPU share that GPU's array: two calls that can
 * overlap in time (different streams, or graphs replayed concurrently) race; calls ordered on one
 * stream do not.
 */
#define FQ_STATIC_SCRATCH_BYTES (1u << 20)
#define FQ_STATIC_MAX_SLOTS 32768
#define FQ_STATIC_MAX_UNITS 98304
fq_status fq_backward_static(const fq_tensor *t, void *hip_stream);

/*
 * The same forward (mode FQ_MODE_FORWARD) or backward (FQ_MODE_BACKWARD) for a whole list
 * of tensors -- e.g. the activations and weights of all 22 quantized convolutions of the
 * front end (Sec. 4.3.4 "Quantization coverage") -- in ONE kernel launch instead of one to three per layer
 * (Sec. 3.3).  `ts` is a host array of n descriptors; it is copied to the start of the
 * workspace on `stream` and may be reused as soon as the call returns.  n = 0 is a no-op.
 * FQ_FLAG_TWO_PASS on any tensor selects the two-launch backward for the whole list.
 *
 * Host-side behaviour of the table copy (also in fq_plan_create and, when the step changes, in
 * fq_plan_run_adam): the table is staged in one of eight pinned host buffers that the library
 * keeps for the life of the process.  A buffer is allocated (hipHostMalloc) the first time it is
 * used or when a larger table comes along, and a call that finds its buffer still being read by a
 * copy enqueued eight such calls earlier waits on the host for that one copy to finish
 * (hipEventSynchronize); no other call of the library ever blocks.  Because of the allocation and
 * the possible wait these three calls must not be made while a stream is being captured into a
 * HIP graph: capture fq_plan_run (or the single-tensor calls) instead.
 */
fq_status fq_multi_tensor(const fq_tensor *ts, int n, int mode,
                          void *workspace, size_t ws_bytes, void *hip_stream);

/*
 * The same multi-tensor launch, prepared once and replayed: the front end's tensor list is
 * static (the same 22 layers every frame, Sec. 4.3.4), so validation, chunk planning and the
 * copy of the descriptor table need not be repeated per call.
 *
 * fq_plan_create validates `ts` exactly as fq_multi_tensor does, copies the descriptor table to
 * the head of `workspace` on `stream` and returns a host-side plan.  fq_plan_run enqueues the
 * kernel(s) on `stream` and nothing else (no copy, no host allocation), so it may be captured in
 * a HIP graph.  The plan keeps the device pointers it was created with: the tensors and the
 * workspace must stay allocated at the same addresses, the workspace must not be written by
 * anything else (one workspace per plan; zero it before fq_plan_create for backward plans), and
 * fq_plan_run must be ordered after fq_plan_create's stream work.  Tensor contents and theta may
 * change freely between runs.  fq_plan_destroy frees the host-side plan only (NULL is allowed).
 *
 * Backward plans whose descriptors carry a fused Adam step: fq_plan_run repeats the step number
 * the plan was created with; fq_plan_run_adam(plan, step, stream) first brings the bias
 * corrections 1-beta^step of every such tensor up to date (one small asynchronous copy of the
 * table on `stream`, skipped when `step` is the one already in place), then launches.  It is the
 * call for a training loop: step = 1, 2, 3, ...  (It does host work beyond the launch, so capture
 * fq_plan_run, not this, in a graph.)
 */
typedef struct fq_plan fq_plan;
fq_status fq_plan_create(const fq_tensor *ts, int n, int mode, void *workspace, size_t ws_bytes,
                         void *hip_stream, fq_plan **plan);
fq_status fq_plan_run(const fq_plan *plan, void *hip_stream);
fq_status fq_plan_run_adam(fq_plan *plan, int64_t step, void *hip_stream);
void fq_plan_destroy(fq_plan *plan);

/*
 * Distillation loss between one student and one teacher feature map, and its gradient with
 * respect to the student (Sec. 3.2, Eq. (7)): the producer of the gy that fq_backward consumes.
 *   mse   = mean over all n*channels*inner elements of (a - b)^2
 *   cos_p = <a_p, b_p> / (max(||a_p||, eps) * max(||b_p||, eps))   per position p = (n, m), the
 *           inner product and the norms running over the channel axis
 *   cosim = mean of cos_p over the n*inner positions
 *   loss  = mse + lambda * (1 - cosim)
 * The paper prints neither lambda nor the axis of the cosine; lambda is a field, and the channel
 * axis is the reading taken (a patch descriptor is the channel vector at one position).
 * Writes out[0..2] = mse, cosim, loss (binary64, device memory) and, if gstudent != NULL,
 * gstudent = upstream * dloss/dstudent in the tensors' dtype (rounded once from binary64; a
 * clamped norm counts as a constant).  `upstream` is the factor in front of this pair's loss in
 * the total (Eq. (7) sums the pairs: 1, or the loss scale of an FP16 run).  student / teacher are
 * contiguous [n, channels, inner]; gstudent may be exactly student or teacher (in place).  Two or
 * three launches; no atomics, fixed summation order.  A tensor without elements needs no workspace and
 * gives NaN for mse and loss (a mean of nothing); cosim is then NaN without positions and 0 with
 * positions but no channels.  The workspace need not be initialised and may be shared with other calls
 * that do not overlap in time.
 */
typedef struct fq_distill {
    int64_t n, channels, inner;
    int32_t dtype;                    /* fq_dtype of student, teacher, gstudent */
    float lambda, eps, upstream;      /* eps >= 0 (1e-8 is customary); no NaN */
    const void *student, *teacher;    /* in */
    void *gstudent;                   /* out, optional */
    double *out;                      /* out: 3 doubles, 8-byte aligned */
} fq_distill;
size_t fq_distill_workspace_bytes(const fq_distill *d);   /* 0 if d does not validate; host only */
/* How often fq_distill_loss reads the pair from memory for this descriptor: 1 (one fused kernel
   holds a tile of the pair in registers from the statistics to the gradient: up to 512 channels,
   inner a multiple of 4, pointers aligned to 4 elements; also when no gradient is asked for) or 2
   (a statistics kernel, then a gradient kernel); 0 if d does not validate or has no elements.
   Pure host function. */
int fq_distill_reads_of_pair(const fq_distill *d);
fq_status fq_distill_loss(const fq_distill *d, void *workspace, size_t ws_bytes, void *hip_stream);

/*
 * Measurement aid, not part of the operation: a streaming kernel without arithmetic in the launch
 * shape of fq_forward / fq_backward (256-thread blocks, 20 KiB of each stream per block, every
 * load issued before the first store, non-temporal), so that a benchmark can put what the memory
 * system and the launch alone take for the same bytes beside the library's own figures.
 *   inputs = 0: the launch alone (blocks that return at once; the pointers are not touched)
 *   inputs = 1: out = a             (the forward's traffic: `bytes` read, `bytes` written)
 *   inputs = 2: out = a XOR b       (the backward's traffic: 2 x `bytes` read, `bytes` written)
 * a, b, out: device pointers, 16-byte aligned, `bytes` (a multiple of 16) each; out may not
 * overlap a or b partially.
 */
fq_status fq_probe_stream(int inputs, const void *a, const void *b, void *out, size_t bytes, void *hip_stream);

/* Static, NUL-terminated description of a status code. */
const char *fq_status_string(fq_status status);

#ifdef __cplusplus
}
#endif
#endif /* FQ_H */
