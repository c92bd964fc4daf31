/*
 * eco.h — C ABI of the ECO optimizer-step library for AMD MI355X (gfx950).
 *
 * ECO ("Error-Compensating Optimizer", paper "ECO: Quantized Training without
 * Full-Precision Master Weights") trains with quantized weights and no
 * high-precision master copy: each step applies the optimizer update directly
 * to the de-quantized weights, re-quantizes, and adds the quantization error,
 * suitably scaled, to the first-moment buffer (Alg. 1: OPTIM_STEP followed by
 * ECO_QUANTIZE; Alg. 2 for SGD with momentum, Alg. 3 for Adam).
 *
 * One call of eco_step() performs, for every scale group ("block") of
 * `block_size` consecutive elements of every tensor of a plan, in one fused
 * pass over memory:
 *     theta^  = dec(code) * scale                         (Sec. 3.1, x^ = s*y)
 *     m~ = b1*m + (1-b1)*g ;  v~ = b2*v + (1-b2)*g*g      (Sec. 3.2 / Eq. m_tilde)
 *     d  = sqrt(v~/(1-b2^k)) + eps
 *     eta_t = (lr/(1-b1^k)) / d ;  theta~ = theta^ - eta_t * m~
 *                                                         (Sec. 3.2: element-wise step size eta_t)
 *     scale' = max|theta~| / rho ;  code' = round(theta~ * rho/max|theta~|)
 *                                                         (Sec. 3.1, Eq. 1 and s = max|x|/rho)
 *     e  = theta~ - dec(code')*scale'                     (Alg. 3 line 2)
 *     m^ = m~ + ((1-b1^k)/lr)(1-1/b1) * d * e             (Alg. 3 line 5);  v^ = v~
 * (ECO_MODE_ECO; see eco_mode_t for the naive, exact-injection and master-weight variants)
 * with `round` either round-to-nearest-even or stochastic rounding driven by a
 * counter-based Philox4x32-10 generator.  For SGD with momentum:
 *     m~ = b*m + (1-b)*g ; theta~ = theta^ - lr*m~ ; m^ = m~ + (1/lr)(1-1/b)*e
 *                                                         (Sec. 3.3.1 Eqs. m_tilde..alpha, Alg. 2)
 *
 * Conventions
 *  - Every data pointer in eco_tensor_t and in the helper calls is a DEVICE
 *    pointer owned by the caller; descriptors and hyper-parameter structs are
 *    HOST memory and are read during the call only.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *    work is enqueued on it; no call synchronizes unless it says so.
 *  - Weights, scales, m and v are updated in place; gradients are only read.
 *  - Every function returns an eco_status_t; nothing aborts or throws.  After a
 *    failure eco_last_error() (thread-local) describes it, and no kernel of
 *    that call has been launched unless the status is ECO_EHIP (a launch that
 *    fails stops the call: kernels enqueued before it still run).  An error
 *    left pending in the HIP runtime by the caller's earlier work is cleared
 *    on entry and not reported.
 *  - Results depend only on the inputs, the hyper-parameters, (seed, step,
 *    tensor_id) and the element index: never on launch geometry, on the order
 *    of tensors in a plan, or on which tensors share a launch.
 *  - Inputs are assumed finite; behaviour on NaN/Inf is unspecified.
 *  - A plan may be used by one host thread at a time; eco_set_option may be
 *    called from any thread.
 *
 * Performance notes for callers (MI355X; none of this changes results)
 *  - The step is bound by HBM bandwidth (the INT4 / bf16-state form by vector-ALU issue) and runs at the rate
 *    of a plain copy kernel on the same arrays.  The arrays of a tensor are streamed in lock-step, and where they
 *    lie in device memory relative to each other matters by 2-3 per cent of the step (9 per cent of its memory
 *    traffic alone): measured inside one allocation of most of the memory, the address space falls into 32 GiB
 *    regions of three kinds, and the step is at its best when m or v lies in a region of another kind than the
 *    other arrays.  Which region is of which kind depends on the physical addresses an allocation gets;
 *    eco_bandwidth_probe, timed on candidate addresses before anything is stored there, tells.
 *  - One plan over all tensors of a model is one kernel launch per storage format; per-tensor calls pay a
 *    launch each.
 *  - Tensor lengths that are multiples of 512 keep every tile on the unguarded fast path.
 *  - Row-wise scale groups (group_size = the row length) of more than 512 elements run with every lane busy when the
 *    row is a multiple of 512 elements, or when 2, 4 or 8 rows together are (576, 640, 768, 1408, 2304, ...) and the
 *    tensor has a multiple of that many rows; other lengths leave part of each row's last wave idle.
 */
#ifndef ECO_H
#define ECO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ECO_OK = 0,
  ECO_EINVAL = -1,        /* null pointer, zero size, step == 0, lr/beta out of range, ... */
  ECO_EALIGN = -2,        /* a data pointer is not 16-byte aligned                          */
  ECO_EUNSUPPORTED = -3,  /* no kernel for this combination (e.g. block size)               */
  ECO_EHIP = -4,          /* a HIP runtime call failed (no device, launch error, ...)       */
  ECO_ENOMEM = -5         /* host or device allocation for a plan failed                    */
} eco_status_t;

/* Storage format of a tensor's weights (Sec. 3.1: the format fixes rho and the code grid). */
typedef enum {
  ECO_FMT_FP8_E4M3 = 0,      /* 1 byte/element, OCP E4M3 (bias 7, max 448, S.1111.111 = NaN, no Inf); rho = 448 */
  ECO_FMT_INT4 = 1,          /* 2 elements/byte, two's complement in [-7,7], element 2j in the low nibble; rho = 7 */
  ECO_FMT_BF16_PLAIN = 2,    /* bfloat16 weights, no quantizer and no injection: ordinary Adam/SGDM (the paper
                                applies the method to linear layers only, Sec. 4.2 "Setting")                      */
  ECO_FMT_FP32_IDENTITY = 3  /* fp32 weights, identity quantizer: e = 0, the step reduces to the plain optimizer   */
} eco_format_t;

typedef enum { ECO_OPT_ADAM = 0, ECO_OPT_SGDM = 1 } eco_opt_t;       /* Alg. 3 / Alg. 2              */
typedef enum { ECO_ROUND_SR = 0, ECO_ROUND_RTN = 1 } eco_round_t;    /* Sec. 3.1, rounding function  */
typedef enum { ECO_DT_FP32 = 0, ECO_DT_BF16 = 1 } eco_dtype_t;

/* What happens to the quantization error e = theta~ - q(theta~). */
typedef enum {
  ECO_MODE_NAIVE = 0,   /* nothing: master weights simply removed (Sec. 4.1 "FP8 w/o MW" baselines)               */
  ECO_MODE_ECO = 1,     /* the paper's method: memory-free injection into m (Alg. 2 line 5 / Alg. 3 line 5)        */
  ECO_MODE_EXACT = 2,   /* SGDM only: exact injection with a stored error, m <- m~ + e_t/eta - e_{t+1}/(eta beta)
                           (Appendix A, Eq. im_inject); reproduces master-weight SGDM, costs 4 bytes/parameter     */
  ECO_MODE_MASTER = 3   /* baseline WITH fp32 master weights (Sec. 3.1; Sec. 4.1 "FP8 w/ MW"): the update is applied
                           to the master copy, weights = q(master), m is left alone                               */
} eco_mode_t;

/* One parameter tensor, flattened row-major.  Element i belongs to scale group i / group_size;
 * the last group may be shorter.  All pointers: device memory, 16-byte aligned. */
typedef struct eco_tensor {
  void *weights;        /* FP8: numel bytes; INT4: ceil(numel/2) bytes; BF16_PLAIN: numel bf16; FP32_IDENTITY: numel fp32 */
  void *scales;         /* ceil(numel/block_size) entries of scale_dtype; ignored (may be NULL) for the last two formats  */
  const void *grad;     /* numel bfloat16, read only                                                                       */
  void *m;              /* first moment, numel entries of state_dtype                                                      */
  void *v;              /* second moment, numel entries of state_dtype; ignored (may be NULL) for ECO_OPT_SGDM             */
  void *aux;            /* numel fp32: ECO_MODE_EXACT: the stored error e_t (in: e_t, out: e_{t+1});
                           ECO_MODE_MASTER: the master weights (in place); ignored (may be NULL) in the other modes        */
  uint64_t numel;       /* > 0                                                                                             */
  uint64_t group_size;  /* elements per scale group (Sec. 3.1 "granularity"); 0 = hparams.block_size.  Supported: powers
                           of two in [32, 512] (block-wise); any multiple of 8 up to 8192 (e.g. the row length: row-wise
                           scaling as in Sec. 4.1); >= numel (one scale for the tensor, as in Sec. 4.4).  The number of
                           scales is ceil(numel / group_size); ignored for the unquantized formats                         */
  uint32_t tensor_id;   /* enters the random-number counter; keep it stable across steps and distinct across tensors      */
  int32_t fmt;          /* eco_format_t                                                                                    */
} eco_tensor_t;

/* Hyper-parameters H of Alg. 1-3 plus the description of the quantizer and of the state layout. */
typedef struct eco_hparams {
  int32_t opt;            /* eco_opt_t                                                                     */
  int32_t round;          /* eco_round_t: rounding used when re-quantizing                                 */
  int32_t mode;           /* eco_mode_t; 1 = ECO                                                           */
  uint32_t block_size;    /* default scale group of the plan's tensors: 32, 64, 128, 256 or 512 elements   */
  int32_t state_dtype;    /* eco_dtype_t of m and v (math is fp32; bf16 state is rounded to nearest even)  */
  int32_t scale_dtype;    /* eco_dtype_t of the scales                                                     */
  double lr;              /* eta  (> 0 when the mode injects)                                              */
  double beta1;           /* beta1, or beta for SGDM (in (0,1) when the mode injects: it divides by beta)  */
  double beta2;           /* beta2 (Adam only, in [0,1))                                                   */
  double eps;             /* epsilon (Adam only, >= 0)                                                     */
  double weight_decay;    /* decoupled decay lambda: theta^ <- theta^ - lr*lambda*theta^ before the update */
  uint64_t step;          /* k >= 1: the 1-based index of the step being taken (bias corrections 1-beta^k) */
  uint64_t seed;          /* key of the stochastic-rounding generator                                      */
} eco_hparams_t;

/* The fp32 constants a step uses, derived from eco_hparams_t in double and rounded once. */
typedef struct eco_constants {
  float b1, omb1, b2, omb2;   /* beta1, 1-beta1, beta2, 1-beta2                     */
  float rbc2;                 /* 1/(1-beta2^k)                                       */
  float c1;                   /* lr/(1-beta1^k)  (Adam);                             */
  float eps;
  float kappa;                /* ((1-beta1^k)/lr)(1-1/beta1)  (Alg. 3 line 5); 0 unless ECO_MODE_ECO */
  float lr;                   /* eta (SGDM)                                          */
  float alpha;                /* (1/lr)(1-1/beta)  (Eq. alpha); 0 unless ECO_MODE_ECO */
  float wd;                   /* lr*lambda                                           */
  float inv_lr;               /* 1/lr          (Appendix A, Eq. im_inject); 0 unless ECO_MODE_EXACT */
  float inv_lr_beta;          /* 1/(lr*beta)                                         */
} eco_constants_t;

typedef struct eco_plan eco_plan_t;

/*
 * eco_plan_create — validate a list of tensors and upload its launch tables (Alg. 1 is applied to
 * every tensor of the list by one eco_step call; tensors of different formats may be mixed).
 *   tensors, n : HOST array of n >= 1 descriptors (copied; may be freed after the call)
 *   layout     : HOST; only block_size, state_dtype, scale_dtype, opt and mode are read (they fix the
 *                memory layout the descriptors are checked against)
 *   out        : receives the plan; owned by the library until eco_plan_destroy
 * Allocates device memory for the tables (80 bytes per tensor + 4 bytes per 512 elements, or per scale group
 * for groups wider than 512; for tensors with a single scale over more than 8192 elements another 4 bytes per
 * 512 elements of scratch) and copies them synchronously.
 * Errors: ECO_EINVAL, ECO_EALIGN, ECO_EUNSUPPORTED, ECO_ENOMEM, ECO_EHIP.
 */
eco_status_t eco_plan_create(const eco_tensor_t *tensors, size_t n, const eco_hparams_t *layout, eco_plan_t **out);

/* Frees the plan's host and device tables (synchronizes the device first).  NULL is allowed. */
eco_status_t eco_plan_destroy(eco_plan_t *plan);

/*
 * eco_step — one ECO step (Alg. 1 with Alg. 3 or Alg. 2) over every tensor of the plan.
 * Asynchronous on `stream`; allocates nothing.  Launches per storage format present: one kernel over the full
 * 512-element tiles of block-scaled tensors, one over their ragged tails if any, one per workgroup size for wide
 * groups, and four for tensors with a single scale (abs-max pass into the plan's scratch, its reduction, apply
 * pass, scale write); a plan with more work than one launch can hold (2^32 threads: about 2^35 elements) has these
 * launched in pieces.  Steps of one plan that use that scratch must not overlap each other on different streams.
 * hp->block_size, state_dtype, scale_dtype, opt and mode must equal the plan's, and the device that was current at
 * eco_plan_create must be current (ECO_EINVAL otherwise).
 */
eco_status_t eco_step(eco_plan_t *plan, const eco_hparams_t *hp, void *stream);

/*
 * eco_step_tensors — convenience form without a persistent plan: builds the tables, runs the step,
 * waits for `stream`, and frees the tables.  Allocates device memory and synchronizes.
 */
eco_status_t eco_step_tensors(const eco_tensor_t *tensors, size_t n, const eco_hparams_t *hp, void *stream);

/*
 * eco_step_tensors_noalloc — eco_step_tensors for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results bit for
 * bit; asynchronous on `stream` (it does not wait for it, unlike eco_step_tensors).  Calls no hipMalloc, hipFree,
 * host-to-device copy or other allocating routine: the tensor descriptors, the launch tables and the abs-max
 * scratch of tensors with a single scale live in one static device array of 8.7 MB (8 732 672 bytes) per GPU,
 * held until the process ends, and the tables are written by a kernel from descriptors passed as kernel arguments.
 * Limits: at most 4096 tensors per call and at most 2^20 launch-table entries in total (one per 512 elements of a
 * tensor, rounded up, plus one per tensor with a ragged tail or a single scale; one per scale group for groups
 * wider than 512 elements) -- about 5.3e8 elements per call; beyond that ECO_EUNSUPPORTED, before anything is
 * launched.  Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (different
 * streams, different host threads) race; calls on one stream, or ordered by events, are safe.  Nothing in the
 * array has to start at zero: every entry a step reads is written earlier in the same call.
 */
eco_status_t eco_step_tensors_noalloc(const eco_tensor_t *tensors, size_t n, const eco_hparams_t *hp, void *stream);

/*
 * eco_quantize_init — q(x) of Sec. 3.1 with round-to-nearest-even, for setting up quantized weights.
 *   src    : device, numel values of src_dtype (ECO_DT_FP32 or ECO_DT_BF16)
 *   weights, scales : device outputs, laid out as in eco_tensor_t
 * fmt must be ECO_FMT_FP8_E4M3 or ECO_FMT_INT4; group_size as in eco_tensor_t (not 0).  Asynchronous on `stream`.
 * With one scale for a tensor of more than 8192 elements the abs-max is kept in a library-owned slot between
 * the call's kernels; the library hands out 64 such slots in turn and makes a call wait, on its own stream, for
 * the previous user of its slot, so calls on different streams may overlap.
 * Size limit, for this call, eco_dequantize and eco_quantize_error alike: what one kernel launch holds (fewer than
 * 2^32 threads, one thread per 8 elements: just under 2^35 elements; less for groups of 520..8192 elements whose
 * length is far from a multiple of 512).  Larger arrays are ECO_EUNSUPPORTED: pass slices of whole scale groups.
 * (eco_step and eco_step_tensors have no such limit: they launch in pieces.)
 */
eco_status_t eco_quantize_init(const void *src, int32_t src_dtype, uint64_t numel, int32_t fmt, uint64_t group_size,
                               int32_t scale_dtype, void *weights, void *scales, void *stream);

/* eco_dequantize — dst[i] = dec(code_i) * scale[i / group_size] as fp32 (Sec. 3.1, x^ = s*y); group_size >= 8,
 * or one group over the whole tensor.
 * Asynchronous. */
eco_status_t eco_dequantize(const void *weights, const void *scales, uint64_t numel, int32_t fmt, uint64_t group_size,
                            int32_t scale_dtype, float *dst, void *stream);

/*
 * eco_quantize_error — err[i] = src[i] - dec(code_i) * scale[i / group_size] as fp32: the quantization error
 * e = theta - q(theta) of Sec. 3.1 (notation paragraph) for weights quantized from `src`.  It is the initial
 * stored error e_0 of the exact-injection mode (Appendix A, Eq. init_im: e_0 = theta_0 - q(theta_0)).
 *   src : device, numel values of src_dtype; weights, scales: device, as written by eco_quantize_init
 *   err : device output, numel fp32, 16-byte aligned
 * group_size >= 8, or one group over the whole tensor.  Asynchronous.
 */
eco_status_t eco_quantize_error(const void *src, int32_t src_dtype, const void *weights, const void *scales, uint64_t numel,
                                int32_t fmt, uint64_t group_size, int32_t scale_dtype, float *err, void *stream);

/*
 * eco_philox_fill — the raw random stream the stochastic rounding of (seed, step, tensor_id) draws from:
 * dst[j] = output word (j & 3) of Philox4x32-10 with key (seed lo, seed hi) and counter
 * ((j>>2) lo, (j>>2) hi, step lo, tensor_id), for j = first_word .. first_word + n_words - 1.
 * Element i of a tensor uses bits 16*(i&1) .. 16*(i&1)+15 of word (i>>3)*4 + ((i&7)>>1).
 * dst: device, n_words uint32.  Asynchronous.
 */
eco_status_t eco_philox_fill(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t first_word, uint64_t n_words,
                             uint32_t *dst, void *stream);

/*
 * eco_bandwidth_probe — measurement aid, not part of the method: what the memory system delivers for the step's
 * access pattern with the arithmetic taken out (the ceiling a step can be compared with; and, timed on candidate
 * addresses before anything is stored there, a way to choose where the arrays should lie, see the performance notes).
 *   kind 0: byte-mix copy.  Every lane loads what a lane of the FP8 / fp32-state Adam step loads for its 8 elements
 *           (codes, gradient, m, v, the 128-block's scale) and stores what it stores, same tile geometry and
 *           occupancy cap: 11.03 B read + 9.03 B written per element.  codes: numel bytes, scales: numel/128 fp32,
 *           grad: numel bf16, m and v: numel fp32.  The contents of codes, m and v are scrambled (m and v swap).
 *   kind 1: plain copy of numel fp32 from m to v (4 B read + 4 B written per element); the other pointers are ignored.
 * numel: a multiple of 1024.  All pointers device, 16-byte aligned.  Asynchronous.
 */
eco_status_t eco_bandwidth_probe(int32_t kind, void *codes, void *scales, const void *grad, void *m, void *v, uint64_t numel,
                                 void *stream);

/*
 * eco_arith_selftest — device self-test of the two short arithmetic sequences of the step kernels.  Inside stated
 * operand ranges the kernels compute the correctly rounded square root (kind 0; arguments in [2^-96, 2^96]) and
 * the correctly rounded quotient numerator / d (kind 1; |numerator| in [2^-40, 2^40], d in [2^-48, 2^49]) with
 * shorter instruction sequences than sqrtf() and `/`; this call compares short and long form for every fp32 bit
 * pattern x (kind 0) or d (kind 1) of [bits_lo, bits_hi) and ADDS the number of patterns on which they differ
 * (expected: 0) to *mismatches (device memory, uint64, 8-byte aligned, cleared by the caller).  Ranges outside
 * the ones above: ECO_EINVAL.  Asynchronous.
 */
eco_status_t eco_arith_selftest(int32_t kind, float numerator, uint32_t bits_lo, uint32_t bits_hi, uint64_t *mismatches,
                                void *stream);

/* eco_step_constants — host only: validates hp as eco_step does and writes the derived fp32 constants. */
eco_status_t eco_step_constants(const eco_hparams_t *hp, eco_constants_t *out);

/* Launch tuning, host only; never changes results.
 *   option 0: cap on the step kernel's grid, in workgroups per compute unit; the kernel then loops over
 *             tiles (0 = library default: one workgroup per 512-element tile, no cap)
 *   option 1: bytes of dynamic LDS requested per workgroup of the step kernel (-1 = library default).
 *             The kernel never touches it; the request only caps resident workgroups per compute unit.
 *   option 2: the same per wave of the wide-group and tensor-wise kernels (-1 = library default)
 *   option 3: most threads one kernel launch of a step may have, in [1024, 2^32 - 1] (-1 = the runtime's limit,
 *             2^32 - 1).  A step with more work items than that launches its kernels in several pieces; a small
 *             value lets a test take that path with a small plan. */
eco_status_t eco_set_option(int32_t option, int64_t value);

const char *eco_status_string(int status);   /* status: an eco_status_t; any other value gives "unknown status" */
const char *eco_last_error(void);   /* thread-local, never NULL */
int eco_version(void);              /* major*10000 + minor*100 + patch */

#ifdef __cplusplus
}
#endif
#endif /* ECO_H */
