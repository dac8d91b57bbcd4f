/*
 * mcf.h - C ABI of the MI355X (gfx950) implementation of the Collage optimizer
 * step (arXiv 2405.03637): AdamW with the weights and, optionally, Adam's
 * second moment kept as two-component bf16 expansions (value, error).
 *
 * Number format and the single operation
 *   bf16 is passed as uint16_t: the upper 16 bits of an IEEE binary32,
 *   little endian.  Every arithmetic step is the paper's bf16 operation
 *   F(a o b) (Sec. 3.1): operands widened exactly to fp32, one fp32 operation,
 *   one round-to-nearest-even to bf16.  Subnormals are kept, infinities and
 *   NaN follow IEEE 754; every NaN result is stored as 0x7FC0.
 *   The paper states its algorithms for any low-precision component and names
 *   fp16 beside bf16 (Sec. 1; App. A Table 7: 5 exponent bits, 10 stored
 *   significand bits).  With the fp16 component the same uint16_t buffers hold
 *   IEEE binary16 patterns, F rounds to fp16, the scalars are cast to fp16, and
 *   every NaN result is stored as 0x7E00.  fp16's range is the caller's
 *   business: an epsilon below 2^-25 becomes 0 and squared gradients below
 *   2^-24 are lost or subnormal, so gradients normally need a loss scale the
 *   paper does not specify; none is applied here.
 *   The two FP8 formats of Table 7 are the paper's "direct extension to 8-bit"
 *   (Sec. 7), read as the same chain once more: buffers of uint8_t, one pattern
 *   per element, passed through the same void pointers.  E5M2 (5 exponent bits,
 *   2 stored significand bits, bias 15) is IEEE-style with infinities; every NaN
 *   result is stored as 0x7E.  E4M3 (4 and 3 bits, bias 7) has no infinities:
 *   its largest number is 448 (0x7E), only S.1111.111 is NaN, and a result that
 *   rounds beyond 448 (an infinite one included) is NaN, stored as 0x7F.  With
 *   3 or 4 significant bits most hyper-parameters are far from their fp64
 *   values (E4M3 turns a learning rate below 2^-10 into 0): the formats are
 *   provided for the arithmetic's sake, and scaling is again the caller's.
 *
 * Conventions for every entry point
 *   - Returns MCF_OK (0) or a negative mcf_status.  No exceptions, no errno,
 *     no logging.  Arguments are validated before the first HIP call, so the
 *     argument errors below are reported even on a machine without a GPU.
 *   - "device" pointers address HIP device memory of the current device and are
 *     OWNED BY THE CALLER: the library never allocates, frees or keeps tensor
 *     memory.  "host" pointers are ordinary process memory, read during the
 *     call only.
 *   - bf16 and fp16 buffers need 2-byte alignment (FP8 buffers none), fp32 buffers 4-byte, double
 *     buffers 8-byte (else MCF_ERR_ALIGN).  Any such alignment is accepted.  The step
 *     and the primitives use 128-bit accesses cut on the first buffer's (theta's) 16-byte grid:
 *     fastest when all buffers of one tensor share the same offset modulo 16 bytes (modulo 1 KiB
 *     for the last 2-4%: buffers shifted against each other by 128 to 512 bytes measured slower); a
 *     buffer at another offset is accessed unaligned, which the hardware splits (the fp32-master
 *     baseline goes element by element instead when its buffers are not mutually aligned).
 *   - Updates are in place.  Buffers of different roles or tensors must not
 *     overlap (not checked; the result is undefined if they do).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it and the call returns without waiting.
 *   - The library owns only plan objects (a host struct, device tables with a
 *     small pinned host staging block for them, and one device buffer of
 *     reduction partials) between create and destroy.
 *   - Calls on one plan must not overlap in time; distinct plans are independent.
 */
#ifndef MCF_H
#define MCF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MCF_OK = 0,
  MCF_ERR_NULL = -1,     /* a required pointer is NULL */
  MCF_ERR_SIZE = -2,     /* a size is out of range (tensor longer than 2^35 - 128 elements, table too large) */
  MCF_ERR_ALIGN = -3,    /* a pointer is not aligned to its element size */
  MCF_ERR_VARIANT = -4,  /* variant is not one of mcf_variant, or an operation code is unknown */
  MCF_ERR_STEP = -5,     /* step < 1 (the bias correction 1 - beta^0 would be zero) */
  MCF_ERR_HYPER = -6,    /* a hyper-parameter is not finite, or beta not in [0,1), or lr/eps/weight_decay < 0 */
  MCF_ERR_HIP = -7       /* a HIP runtime call failed (no device, out of memory, launch failure) */
} mcf_status;

/* Text for a status code; never NULL. */
const char *mcf_status_string(int status);

/* Alg. 2 line 1: learning rate alpha, beta1, beta2, epsilon, weight decay lambda.
 * The library derives the bf16 scalars itself, in fp64, each cast once
 * (App. D "Scalar and Bias Correction"): beta1, 1-beta1, beta2 (plus: its
 * two-component expansion, Table 2), 1-beta2, 1-beta1^t, 1-beta2^t, eps,
 * lambda, -alpha. */
typedef struct { double lr, beta1, beta2, eps, weight_decay; } mcf_hyper;

/* Sec. 4.2: light = expansion for the parameters only (option B, 10 bytes of state
 * per parameter with the gradient); plus = also for the second moment (option C).
 * The other two are the paper's comparison strategies on the same chain (lines 8-12
 * unchanged): MCF_BF16 = plain bf16, option A, line 13 is Eq. 1 theta <- F(theta + delta);
 * MCF_KAHAN = Kahan-compensated bf16 (App. B): u = F(delta + c), theta' = F(theta + u),
 * c <- F(u - F(theta' - theta)), with c kept in dtheta.
 * MCF_SGD = SGD with momentum on the parameter expansion (Sec. 1 calls the extension
 * straightforward and prints no algorithm; the reading here keeps Alg. 2's two changes: the decay
 * term inside the summed update and Grow): m <- F(F(mu*m) + g), delta <- F(-lr * F(m + F(wd*theta))),
 * (theta,dtheta) <- Grow((theta,dtheta), delta); mu = hyper.beta1, hyper.beta2 and hyper.eps are
 * ignored, v and dv are unused and may be NULL. */
typedef enum { MCF_LIGHT = 0, MCF_PLUS = 1, MCF_BF16 = 2, MCF_KAHAN = 3, MCF_SGD = 4 } mcf_variant;
/* May be OR-ed onto MCF_LIGHT or MCF_PLUS: every Grow (Alg. 1) is built on TwoSum (Alg. 3, six
 * operations) instead of Fast2Sum (three), which removes Alg. 1's precondition |x| >= |a| -- it can
 * fail for parameters near zero, for v = 0 at the first step, and when a gradient spike exceeds v
 * (App. C: the same expansion without the ordering).  Any other combination is MCF_ERR_VARIANT. */
#define MCF_GROW_TWOSUM 0x100
/* May be OR-ed onto any variant but MCF_SGD: the denominator of line 12 is F(sqrt(F(v_hat + eps))), epsilon
 * under the root sign as Alg. 2 prints it, instead of the default F(F(sqrt(v_hat)) + eps) of the AdamW the
 * paper says it modifies. */
#define MCF_EPS_INSIDE_SQRT 0x200
/* Component format argument of the primitives below. */
typedef enum { MCF_COMPONENT_BF16 = 0, MCF_COMPONENT_FP16 = 1, MCF_COMPONENT_FP8_E5M2 = 2, MCF_COMPONENT_FP8_E4M3 = 3 } mcf_component;
/* One of these may be OR-ed onto any variant (and combined with MCF_GROW_TWOSUM where that is allowed):
 * the tensors and the derived scalars are of that component format (mcf_component << 12) instead of bf16. */
#define MCF_FMT_FP16 0x1000
#define MCF_FMT_FP8_E5M2 0x2000
#define MCF_FMT_FP8_E4M3 0x3000

/* One parameter tensor: flat, contiguous, n elements per buffer, all device memory.
 * theta, dtheta: the parameter expansion (Alg. 2 lines 2-3; MCF_KAHAN: the Kahan variable;
 * MCF_BF16: unused, may be NULL); m, v: moments;
 * dv: second component of v (MCF_PLUS only, otherwise ignored and may be NULL);
 * grad: this step's gradient, read only. */
typedef struct {
  void *theta, *dtheta, *m, *v, *dv;     /* uint16_t elements (bf16, fp16) or uint8_t elements (FP8) */
  const void *grad;
  uint64_t n;
} mcf_tensor;

typedef struct mcf_plan mcf_plan;

/* Build the launch table for a list of tensors so that one kernel launch steps all of
 * them, however many and however small.  `tensors` is a host array of `count` entries,
 * copied; the device buffers it names must stay valid while the plan is used.  Tensors
 * with n == 0 are allowed and skipped; count == 0 gives a plan whose step does nothing.
 * Allocates device memory for the table (MCF_ERR_HIP if that fails) on the device that is current
 * during the call; the plan belongs to that device, and mcf_plan_update and mcf_adamw_step return
 * MCF_ERR_HIP, launching nothing, when another device is current. */
int mcf_plan_create(mcf_plan **out, const mcf_tensor *tensors, uint32_t count, int variant);
int mcf_plan_destroy(mcf_plan *plan);      /* NULL is accepted */
/* Number of parameters the plan covers (0 for NULL). */
uint64_t mcf_plan_params(const mcf_plan *plan);

/* Point an existing plan at other buffers of the same sizes (for callers whose gradient or parameter
 * buffers are reallocated between steps) without rebuilding it: no allocation.  `tensors` must
 * have the `count` of mcf_plan_create, every n unchanged (else MCF_ERR_SIZE), and each tensor's
 * theta must sit at the same offset modulo 128 bytes as the theta it replaces (else MCF_ERR_ALIGN:
 * the plan's work split was cut for that offset; create a new plan).  Asynchronous like the step: the new
 * table is staged in pinned host memory owned by the plan and copied in `stream` order, behind the steps
 * already enqueued there, into the one of the plan's two device tables that those steps do not read; the
 * call returns without waiting for the copy, and steps enqueued after it use the new buffers.  (The host
 * only waits if it runs two updates ahead of the device: the staging block of the update before the
 * previous one must have been copied.)  `tensors` is read during the call only.  Not for use while
 * `stream` is being captured into a graph (MCF_ERR_HIP): a captured copy would be replayed from whatever
 * the staging memory holds later.  On an error the plan is unchanged. */
int mcf_plan_update(mcf_plan *plan, const mcf_tensor *tensors, uint32_t count, void *stream);

/* One optimizer step, Alg. 2 lines 8-13, over every tensor of the plan: one launch.
 * step = t >= 1.  edq_dev: NULL, or a device pointer to 4 doubles that receive, in
 * stream order, {EDQ, S1, S2, LOST} for this step over all parameters of the plan, where
 * S1 = sum delta*effective, S2 = sum delta^2, EDQ = S1/sqrt(S2) (0 if S2 = 0)
 * (Def. 3.3, Eq. 2-3, with the effective update taken on the value theta+dtheta; on theta
 * alone for MCF_BF16), and LOST = the number of parameters with delta != 0 whose value did
 * not change (lost arithmetic, Def. 3.2; LOST/n is the imprecision percentage of Sec. 5.1). */
int mcf_adamw_step(mcf_plan *plan, const mcf_hyper *hyper, uint64_t step, void *stream, double *edq_dev);

/* The ten scalars a step derives from the hyper-parameters (Alg. 2 line 1, Table 2, App. D
 * "Scalar and Bias Correction"), as 16-bit patterns of the component format, written to the host
 * array out[10] in this order: beta1, 1-beta1, beta2 (first component of its expansion), the
 * second component beta2 - first, 1-beta2, 1-beta1^step, 1-beta2^step, eps, weight_decay, -lr
 * (FP8 patterns in the low byte).
 * Each is computed in fp64 and cast once.  Host-only: no GPU is touched.  restricted_mode_ok (may be
 * NULL) receives 1 when the step kernels may use their reciprocal-based arithmetic for these scalars
 * and 0 when they will use the slower exact sequences (bf16: bias corrections below 2^-60, or a non-zero
 * epsilon outside [2^-100, 2^60]; FP8 E5M2: a bias correction of +-2^-16, whose reciprocal is no fp16
 * number); the results are the same bits either way. */
int mcf_step_scalars(int component, const mcf_hyper *hyper, uint64_t step, uint16_t *out, int *restricted_mode_ok);

/* The same step over a single flat tensor, no plan, no allocation.  n == 0 is a no-op. */
int mcf_adamw_step_flat(void *theta, void *dtheta, void *m, void *v, void *dv,
                        const void *grad, uint64_t n, int variant, const mcf_hyper *hyper,
                        uint64_t step, void *stream);

/* ---- primitives (element-wise over n elements, device buffers) ---- */
/* Thm 4.1 (Fast2Sum): x = F(a+b), y = F(b - F(x-a)); exact when |a| >= |b|. */
int mcf_fast2sum(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *y, uint64_t n, void *stream);
/* Alg. 3 (TwoSum): the same expansion in six operations, no ordering needed. */
int mcf_two_sum(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *y, uint64_t n, void *stream);
/* Alg. 1 (Grow): (x,y) <- Grow((x,y), a), in place. */
int mcf_grow(uint16_t *x, uint16_t *y, const uint16_t *a, uint64_t n, void *stream);
/* Alg. 1 built on TwoSum instead of Fast2Sum (no |x| >= |a| precondition), in place. */
int mcf_grow_two_sum(uint16_t *x, uint16_t *y, const uint16_t *a, uint64_t n, void *stream);
/* Alg. 6 (TwoProdFMA): x = F(a*b), e = F(fma(a, b, -x)); x + e = a*b exactly. */
int mcf_two_prod_fma(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *e, uint64_t n, void *stream);
/* Alg. 7 (Scaling): (x,e) = v * (a1,a2): TwoProdFMA(a1,v); e = F(F(a2*v) + e); Fast2Sum(x,e). */
int mcf_scaling(const uint16_t *v, const uint16_t *a1, const uint16_t *a2, uint16_t *x, uint16_t *e, uint64_t n, void *stream);
/* Alg. 8 (Mul): (x,e) = (a1,a2) * (b1,b2): TwoProdFMA(a1,b1); e = F(e + F(F(a1*b2) + F(a2*b1))); Fast2Sum(x,e). */
int mcf_mul(const uint16_t *a1, const uint16_t *a2, const uint16_t *b1, const uint16_t *b2, uint16_t *x, uint16_t *e,
            uint64_t n, void *stream);
/* Sec. 3.1: out = F(a op b) with op 0 add, 1 sub, 2 mul, 3 div, 4 sqrt(a) (b unused, may be NULL). */
int mcf_bf16_op(int op, const uint16_t *a, const uint16_t *b, uint16_t *out, uint64_t n, void *stream);
/* The rounding inside F: out = bf16(in), round-to-nearest-even, in = fp32 device buffer. */
int mcf_round_f32(const float *in, uint16_t *out, uint64_t n, void *stream);

/* The primitives above for either component format (Sec. 1, App. A Table 7); the bf16 names are
 * these with MCF_COMPONENT_BF16.  An unknown component or code is MCF_ERR_VARIANT.
 * mcf_primitive: `which` selects the algorithm and fixes the inputs; the two results go to
 * (o0, o1), which may be the same buffers as (p0, p1) (Grow in place) but must not otherwise
 * overlap an input; unused inputs may be NULL. */
typedef enum {
  MCF_PRIM_FAST2SUM = 0,     /* Thm 4.1: (o0,o1) = Fast2Sum(p0, p1)               */
  MCF_PRIM_TWOSUM = 1,       /* Alg. 3:  (o0,o1) = TwoSum(p0, p1)                 */
  MCF_PRIM_GROW = 2,         /* Alg. 1:  (o0,o1) = Grow((p0,p1), p2)              */
  MCF_PRIM_GROW_TWOSUM = 3,  /* Alg. 1 on Alg. 3                                  */
  MCF_PRIM_TWOPROD = 4,      /* Alg. 6:  (o0,o1) = TwoProdFMA(p0, p1)             */
  MCF_PRIM_SCALING = 5,      /* Alg. 7:  (o0,o1) = p0 * (p1,p2)                   */
  MCF_PRIM_MUL = 6           /* Alg. 8:  (o0,o1) = (p0,p1) * (p2,p3)              */
} mcf_primitive_code;
int mcf_primitive(int component, int which, const void *p0, const void *p1, const void *p2, const void *p3,
                  void *o0, void *o1, uint64_t n, void *stream);
/* Sec. 3.1: out = F(a op b) in the given component format, op as in mcf_bf16_op. */
int mcf_component_op(int component, int op, const void *a, const void *b, void *out, uint64_t n, void *stream);
/* The rounding inside F for the given component format: fp32 device buffer -> 16- or 8-bit patterns. */
int mcf_round_f32_to(int component, const float *in, void *out, uint64_t n, void *stream);

/* Def. 3.3 as a stand-alone reduction: delta = intended update, (th0,dth0) the parameter
 * before and (th1,dth1) after the step; dth0/dth1 may be NULL (plain bf16 parameters,
 * Eq. 2 as printed).  edq_dev as in mcf_adamw_step.  scratch_dev: device buffer of at
 * least mcf_edq_scratch_bytes(n) bytes, 8-byte aligned, used for reduction partials. */
uint64_t mcf_edq_scratch_bytes(uint64_t n);
int mcf_edq(const uint16_t *delta, const uint16_t *th0, const uint16_t *dth0, const uint16_t *th1,
            const uint16_t *dth1, uint64_t n, void *scratch_dev, void *stream, double *edq_dev);
/* The same reduction over buffers of the given component format. */
int mcf_edq_component(int component, const void *delta, const void *th0, const void *dth0, const void *th1,
                      const void *dth1, uint64_t n, void *scratch_dev, void *stream, double *edq_dev);
/* mcf_edq_component for callers that cannot allocate device memory or pass a workspace: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without
 * scratch_dev, same kernels, same results: the reduction partials live in a fixed array inside the
 * library's device code (3.2 MB, held by every GPU the library runs on until the process ends), which
 * bounds n at 2^28 elements (larger: MCF_ERR_SIZE; reduce in pieces, or use mcf_edq_component).  The call
 * allocates and frees nothing.  Its first call on a device looks up that device's copy of the array (no
 * allocation either; make that first call outside a capture).  All calls on one GPU share the one array:
 * calls that overlap in time there, on different streams or from different threads, race on it and give
 * wrong sums; calls on one stream, or otherwise ordered, are fine, and nothing has to be cleared between
 * them. */
int mcf_edq_noalloc(int component, const void *delta, const void *th0, const void *dth0, const void *th1,
                    const void *dth1, uint64_t n, void *stream, double *edq_dev);

/* ---- option D, the mixed-precision baseline the paper compares against (Sec. 2.1, Table 1):
 * bf16 parameter and gradient, fp32 moments and fp32 master weight; plain fp32 AdamW with the
 * same formula as Alg. 2 lines 8-12, master += delta, theta = bf16(master). ---- */
typedef struct {
  uint16_t *theta;          /* written only */
  float *master, *m, *v;
  const uint16_t *grad;
  uint64_t n;
} mcf_fp32mw_tensor;
typedef struct mcf_fp32mw_plan mcf_fp32mw_plan;
/* Plans of the baseline belong to the device current at creation, like mcf_plan. */
int mcf_fp32mw_plan_create(mcf_fp32mw_plan **out, const mcf_fp32mw_tensor *tensors, uint32_t count);
int mcf_fp32mw_plan_destroy(mcf_fp32mw_plan *plan);
int mcf_fp32mw_step(mcf_fp32mw_plan *plan, const mcf_hyper *hyper, uint64_t step, void *stream);

/* ---- measurement aid: a plain 128-bit copy of `bytes` bytes (multiple of 16, both pointers 16-byte
 * aligned device memory, not overlapping) in the step kernel's launch shape.  It is the streaming
 * ceiling the step's bandwidth is reported against and the known-size transfer used to calibrate
 * profiler byte counters (the step moves 18 or 22 bytes per parameter: Table 1's state, read and
 * written, plus the gradient). ---- */
int mcf_stream_copy(void *dst, const void *src, uint64_t bytes, void *stream);
/* ---- tuning aid: override, for every later step launch of this process, how the step kernels pace their
 * memory traffic.  groups_per_cu: single-wave workgroups resident per compute unit (0 = no cap); head_sleep,
 * tail_sleep: s_sleep units (64 clocks each) that every wave idles before its first load and after its last store.
 * A negative value restores the built-in figure of each variant (the caps measured on MI355X at the
 * 7B-parameter set; no sleeps).  Results do not depend on any of this, only the time does.  Values above 128
 * groups or 4096 units are MCF_ERR_SIZE.  Not synchronised with launches on other threads. ---- */
int mcf_set_launch_pacing(int groups_per_cu, int head_sleep, int tail_sleep);

/* ---- measurement aid: the memory traffic of a step without its arithmetic.  Every 16 bytes of each of the
 * n_read buffers reads[] (host array of device pointers, 16-byte aligned, `bytes` bytes each, a multiple of
 * 16) are loaded, and write j (j < n_write <= n_read) receives what read j brought in -- unchanged, so passing
 * the same buffers for reads and writes, as the step does, leaves their contents as they are.  The launch
 * shape is the caller's: threads per workgroup (64 or 256), 128-bit vectors per lane (1, 2 or 4; each wave
 * instruction covers one contiguous run), groups_per_cu, a cap on the workgroups resident per compute
 * unit (0 = none), and store_policy, how the stores are marked for the caches: 0 non-temporal, 1 agent scope
 * (written through to memory), 2 both -- the step kernels use 1, 2 with the EDQ sums fused in, 0 for FP8.
 * Supported mixes (n_read, n_write): (1,1) a copy, (1,0), (4,3), (5,4) the light step,
 * (6,5) the plus step; others are MCF_ERR_VARIANT.  bench.py reports the step against what this reaches. ---- */
int mcf_stream_mix(const void *const *reads, uint32_t n_read, void *const *writes, uint32_t n_write, uint64_t bytes,
                   uint32_t threads, uint32_t vectors_per_lane, uint32_t groups_per_cu, uint32_t store_policy, void *stream);

#ifdef __cplusplus
}
#endif
#endif
