/*
 * coat.h -- C ABI of the MI355X (gfx950) implementation of COAT's FP8-state AdamW step
 * (arxiv 2410.19313: Sec. 3 "Preliminaries", Sec. 4 "Dynamic range expansion",
 * Appendix A "Details about optimizer states quantization") and of the activation quantizers of
 * Sec. 5.2 (1xG per-group, and per-tensor with Group Scaling).
 *
 * Conventions shared by every entry point
 *   - Every data pointer is caller-owned DEVICE memory on the current HIP device.  The
 *     library allocates nothing, keeps no state between calls and frees nothing (one entry point,
 *     coat_act_quant_tensor_static, works in a small device array of the library's own: see there).
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work on that stream; the caller synchronizes.
 *   - A tensor is a flat buffer of n elements.  Every G consecutive elements form one
 *     quantization group (Sec. 3, optimizer state quantization); the last group is short
 *     when n % G != 0.  Per-group arrays have ceil(n/G) entries.
 *   - Base pointers of per-element arrays must be 16-byte aligned; the per-group arrays of the
 *     optimizer state (scale, k) need 4-byte alignment only, so that a shard may start at any even
 *     group (see coat_shard_range).  n is 64-bit (the 7B and 13B parameter sets exceed 2^32
 *     elements).
 *   - Return value: COAT_OK (0) or a negative COAT_ERR_* code.  Arguments are validated on
 *     the host before anything is launched, so a failing call has touched no memory.
 *     n == 0 is a successful no-op.  No exception or abort crosses this boundary.
 *   - FP8 formats: OCP E4M3 (1-4-3 bits, bias 7, max 448, min subnormal 2^-9, no infinity;
 *     0x7F/0xFF are NaN) by default, OCP E5M2 (1-5-2 bits, bias 15, max 57344, min subnormal
 *     2^-16, 0x7C infinity) per moment on request.  Non-finite codes are never produced from
 *     finite inputs.
 *   - Optimizer state: any finite codes with scales and exponents in range are accepted.  The
 *     accuracy the tests state (scales and exponents to 1e-6 of a double-precision evaluation)
 *     is that of states this library writes, in which every non-empty group holds a code of
 *     magnitude fmax (the next one below at most with bf16 scales).  In a hand-made state whose
 *     largest second-moment code of a group is far below fmax, the new scale of that group
 *     inherits the relative error of the inverse expansion at that code (measured: up to 1.3e-6
 *     when no code exceeds 0x30, 8e-7 for 0x50), unless COAT_FLAG_PRECISE_DQ is set (3.6e-7).
 */
#ifndef COAT_H
#define COAT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define COAT_OK            0
#define COAT_ERR_NULL     -1  /* a required pointer is NULL */
#define COAT_ERR_ALIGN    -2  /* a base pointer is not aligned as required (16 bytes; 4 for scale and k) */
#define COAT_ERR_GROUP    -3  /* group size not one of 32, 64, 128, 256, 512 (activation quantizers: or 16) */
#define COAT_ERR_STEP     -4  /* step < 1 */
#define COAT_ERR_HPARAM   -5  /* non-finite or out-of-domain hyper-parameter, unknown flag bit */
#define COAT_ERR_LAUNCH   -6  /* the HIP runtime refused the launch */
#define COAT_ERR_SIZE     -7  /* n exceeds what the launch geometry supports, or a buffer is too small */
#define COAT_ERR_PLAN     -8  /* not a plan blob written by coat_multi_plan_build */

/* Flags.  The per-moment bits select a cell of the paper's Table 1 (each moment stored as E4M3 or
 * E5M2, with or without the expansion); the default (COAT_FLAG_EXPAND alone) is the method as
 * the paper runs it and has its own tuned kernel. */
#define COAT_FLAG_EXPAND   1u  /* dynamic range expansion on (off => k == 1 for both moments) */
#define COAT_FLAG_M_E5M2   2u  /* first moment stored as OCP E5M2 instead of E4M3 */
#define COAT_FLAG_E5M2     2u  /* the same bit, for coat_quant_group / coat_dequant_group */
#define COAT_FLAG_V_E5M2   4u  /* second moment stored as OCP E5M2 */
#define COAT_FLAG_M_PLAIN  8u  /* first moment without expansion even when COAT_FLAG_EXPAND is set */
#define COAT_FLAG_V_PLAIN 16u  /* second moment without expansion even when COAT_FLAG_EXPAND is set */
#define COAT_FLAG_BF16_SCALE 32u /* the per-group scale arrays hold bf16 (uint16_t) values instead of
                                    fp32, as Sec. 3 stores them.  The scale is amax/fmax rounded UP to
                                    a bf16 value, quantizer and dequantizer both use the stored value,
                                    and k is chosen from (fmax*scale)/amin, the range the normalized
                                    group really spans.  Resident state: 8 + 12/G bytes per parameter
                                    instead of 8 + 16/G. */
#define COAT_FLAG_PRECISE_DQ 128u /* dequantize the old moments with the rounding of the exponent log2(c/fmax)/k
                                    recovered (three more instructions per element; about 2.5 % more time on a
                                    7B-parameter step).  The weight update m/(sqrt(v)+eps) inherits the moments'
                                    relative error (up to 2e-6 without this); that stays below 1e-6 of the
                                    WEIGHT for lr = 3e-4, beta = 0.9/0.95, but not when the update is a large
                                    fraction of the weight.  The step therefore takes this path BY ITSELF when
                                    lr * (1 - beta1) / sqrt(1 - beta2), the largest update Adam can make, is
                                    2e-4 or more (PyTorch's defaults lr = 1e-3, beta = 0.9/0.999: 3.2e-3); the
                                    flag asks for it below that.  Codes, scales and exponents do not depend on
                                    it beyond rounding. */
#define COAT_FLAG_BF16_K  64u  /* the per-group exponent arrays hold bf16 (uint16_t) values too: Sec. 4.2
                                  computes k per group and step and keeps it beside the scale.  The
                                  stored k is the clamped exponent rounded to the NEAREST bf16 value
                                  (ties to even, as a cast does), and quantizer and dequantizer both use
                                  the stored value.  R_X^k may then exceed R_format by a factor
                                  R_format^(2^-8); the smallest element still rounds to the smallest
                                  subnormal.  A group that receives no gradient keeps its exponent.
                                  With both flags: 8 + 8/G bytes per parameter. */

/* Hyper-parameters of one step: symbols of Sec. 3, Eq. (1). */
typedef struct {
  float    lr;            /* eta > 0 or 0 */
  float    beta1, beta2;  /* in [0, 1) */
  float    eps;           /* epsilon >= 0, added to sqrt(v_hat) */
  float    weight_decay;  /* lambda, decoupled: enters as eta * lambda * w */
  int32_t  step;          /* t >= 1; bias corrections 1 - beta^t are formed on the host in fp64 */
  int32_t  group_size;    /* G in {32, 64, 128, 256, 512} */
  uint32_t flags;         /* COAT_FLAG_* */
  float    k_min, k_max;  /* clamp applied to the expansion exponent k; 0,0 => 2^-4 and 2^10;
                             otherwise 2^-6 <= k_min <= k_max <= 2^16 */
} coat_adamw_hparams;

/*
 * One fused optimizer step over a flat parameter buffer (Appendix A; kernel structure of
 * Appendix F.4 re-designed for 64-wide wavefronts):
 *   m = DQ(m_q), v = DQ(v_q) with the inverse expansion |.|^(1/k) (Sec. 4.2);
 *   m_t = beta1 m + (1-beta1) g,  v_t = beta2 v + (1-beta2) g^2           (Sec. 3);
 *   w  <- w - lr * ( (m_t/(1-beta1^t)) / (sqrt(v_t/(1-beta2^t)) + eps) + weight_decay * w )  (Eq. 1),
 *        computed from the new moments BEFORE they are quantized;
 *   per group and per moment: amax, amin over non-zero magnitudes (Definition 1),
 *   scale = amax/448, k = log2(448*512)/log2(amax/amin) clamped to [k_min, k_max],
 *   code = E4M3_rne( sign(x) * 448 * (|x| / (448*scale))^k ).
 *
 * w          [n]   fp32 master weights, updated in place.
 * grad_bf16  [n]   bf16 gradients (raw 16-bit patterns), read only.
 * m_q, v_q   [n]   E4M3 codes of the first and second moment, updated in place.
 * m_scale, m_k, v_scale, v_k  [ceil(n/G)]  per-group scale and exponent, in place: fp32, except that
 *              with COAT_FLAG_BF16_SCALE the two scale arrays, and with COAT_FLAG_BF16_K the two
 *              exponent arrays, hold bf16 (uint16_t) values.
 * With COAT_FLAG_*_E5M2 the constants 448 and 448*512 become 57344 and 57344*65536 for that
 * moment; a moment stored without expansion uses the plain quantizer of Sec. 3 (code =
 * round(x/scale), x = scale*code), writes k = 1 and does not read k.
 * The valid start state (m0 = v0 = 0) is: all codes 0, scale 0, k 1.
 * Gradients that are NaN/Inf poison their own element of w and their own group's
 * moments; other groups are unaffected.  Magnitudes below the smallest normal fp32 number (a squared
 * gradient of 1e-20, say) are outside the domain the results are specified for: such an element may
 * count as zero or not; its group's stored state stays valid (finite scale, k within its bounds, no
 * NaN code) and no other group is affected.  A group whose scale amax / fmax would itself fall below
 * the smallest normal fp32 number is stored as the zero state (codes 0, scale 0, k 1).
 */
int coat_fp8_adamw_step(float* w, const uint16_t* grad_bf16,
                        uint8_t* m_q, void* m_scale, void* m_k,
                        uint8_t* v_q, void* v_scale, void* v_k,
                        uint64_t n, const coat_adamw_hparams* hp, void* hip_stream);

/*
 * The same step that ALSO writes the new weights rounded to bf16 (nearest even) into
 * w_bf16 [n]: the copy a mixed-precision trainer hands to its BF16/FP8 model (the paper trains
 * such models from FP32 master weights: Sec. 2, Appendix A), produced in the same pass instead of
 * by a separate cast kernel (+2 bytes written per parameter).  w_bf16 must be 16-byte aligned
 * and must not overlap the other buffers; NULL makes this call identical to coat_fp8_adamw_step.
 */
int coat_fp8_adamw_step_bf16w(float* w, uint16_t* w_bf16, const uint16_t* grad_bf16,
                              uint8_t* m_q, void* m_scale, void* m_k,
                              uint8_t* v_q, void* v_scale, void* v_k,
                              uint64_t n, const coat_adamw_hparams* hp, void* hip_stream);

/*
 * Many tensors in one launch.  A model's parameters are hundreds of separate tensors, many of
 * them small (norm weights, biases); stepping them one call each costs a launch per tensor.  The
 * paper's optimizer treats every tensor alike (Sec. 3: groups of G consecutive elements, each
 * tensor on its own), so the multi-tensor step is the single-tensor step applied to each entry:
 * groups never span two tensors, a tensor's last group is short when n % G != 0, and results are
 * bit-identical to one coat_fp8_adamw_step_bf16w call per tensor with that tensor's weight decay.
 *
 * coat_tensor_desc: the arguments of coat_fp8_adamw_step_bf16w for one tensor (device pointers,
 * same alignment rules; w_bf16 may be NULL) plus its own weight decay (decay / no-decay parameter
 * groups); hp->weight_decay is ignored by the multi-tensor step.  n == 0 entries are skipped.
 *
 * Usage: 1. size a HOST buffer with coat_multi_plan_bytes and fill it with coat_multi_plan_build
 * (pure host code: pointers are validated, never dereferenced).  The blob is a 128-byte header
 * followed by one 128-byte record per span of 32 chunks (32768 elements) of every tensor, each
 * tensor starting a new span: 4 bytes of plan per 1024 elements, plus up to one span of padding
 * per tensor;  2. copy the blob to device memory (16-byte aligned; 128 keeps every record in one
 * cache line);  3. call coat_fp8_adamw_step_multi every step with both copies (the host copy's
 * header gives the launch size, the kernels read the device copy).  The plan stays valid while
 * the tensors' addresses and sizes do; it does not depend on the hyper-parameters or on G.  To
 * step only a shard of a tensor, describe the shard (see coat_shard_range).
 * coat_multi_plan_bytes returns 0 on an invalid argument (NULL with count > 0, an n above 2^46, or
 * 2^21 or more spans in total: one launch covers every span with eight workgroups and a launch
 * holds fewer than 2^24 workgroups).
 */
typedef struct {
  float*          w;
  uint16_t*       w_bf16;        /* optional bf16 copy of the new weights, or NULL */
  const uint16_t* grad_bf16;
  uint8_t*        m_q;  void*  m_scale;  void*  m_k;   /* float[]; uint16_t[] (bf16) with COAT_FLAG_BF16_SCALE / _K */
  uint8_t*        v_q;  void*  v_scale;  void*  v_k;
  uint64_t        n;
  float           weight_decay;  /* lambda of this tensor */
  uint32_t        reserved;      /* set to 0 */
} coat_tensor_desc;

size_t coat_multi_plan_bytes(const coat_tensor_desc* descs, uint32_t count);
int coat_multi_plan_build(const coat_tensor_desc* descs, uint32_t count, void* plan_host, size_t plan_bytes);
int coat_fp8_adamw_step_multi(const void* plan_host, const void* plan_device,
                              const coat_adamw_hparams* hp, void* hip_stream);

/*
 * The multi-tensor step for callers that REPLAY a captured graph across steps.  Kernel arguments
 * are frozen at capture, but three numbers change every step (Sec. 3, Eq. 1: the learning rate of
 * the schedule and the two bias corrections 1 - beta^t; the kernels use them folded into the
 * denominator of the update, see the fields below).  This variant reads them from
 * consts_device, a coat_step_consts in device memory (16-byte aligned) that the caller rewrites
 * between replays with what coat_step_consts_compute (pure host code) returns for the new step;
 * hp->lr, hp->step and hp->eps are validated but not used by the kernels, every other field of hp
 * is frozen into the launch as usual -- the choice of the inverse expansion too: it is made from
 * hp->lr as given at capture (see COAT_FLAG_PRECISE_DQ), so a schedule that crosses that bound
 * should set the flag.  Results are bit-identical to coat_fp8_adamw_step_multi called with the
 * same hyper-parameters and the same choice.
 */
typedef struct {
  float    denom_mul;     /* sqrt((1 - beta2) / (1 - beta2^t)) / c,  c = -lr (1 - beta1) / (1 - beta1^t) */
  float    denom_add;     /* eps / c;  lr == 0 gives denom_mul = 0 and denom_add = +inf (no update) */
  double   neg_lr;        /* -lr */
  uint64_t reserved[2];
} coat_step_consts;

int coat_step_consts_compute(const coat_adamw_hparams* hp, coat_step_consts* out_host);
int coat_fp8_adamw_step_multi_consts(const void* plan_host, const void* plan_device,
                                     const coat_adamw_hparams* hp,
                                     const coat_step_consts* consts_device, void* hip_stream);

/*
 * The shape of the main launch of a single-tensor step over n elements (pure host code): one
 * 1024-element chunk per wavefront, 256 threads per workgroup, and at most 2^24 - 1 workgroups (a
 * dispatch counts its work-items in 32 bits); beyond that many chunks the kernels loop.  For callers
 * that size graphs or occupancy estimates; the ragged last chunk is a second one-wavefront launch.
 */
int coat_launch_shape(uint64_t n, uint32_t* blocks, uint32_t* threads_per_block);

/*
 * The part of a flat tensor of n elements that rank `rank` of `world` owns when optimizer states
 * are sharded (ZeRO / FSDP style; Sec. 3: every rank quantizes its own shard with its own
 * statistics): shards are contiguous, cut at multiples of 2 G (pairs of groups: no group spans two
 * ranks, and a shard's per-group arrays start on a 32-bit word also when the scales are bf16), and
 * differ by at most one pair of groups.  Pure host code.  Writes [*begin, *end); an empty shard has
 * *begin == *end.  Offsetting the element pointers by *begin and the per-group pointers by
 * *begin / G describes the shard to the optimizer step, the multi-tensor plan, coat_quant_group and
 * coat_dequant_group (whose per-group arrays need 4-byte alignment only).
 */
int coat_shard_range(uint64_t n, int32_t G, uint32_t rank, uint32_t world, uint64_t* begin, uint64_t* end);

/*
 * Per-group quantizer with dynamic range expansion (Sec. 3 quantizer Q applied to f(X),
 * Sec. 4.2): the second half of the step on its own.
 * x [n] fp32 in;  q [n] codes, scale/k [ceil(n/G)] out.  All-zero group: scale 0, k 1.
 * flags: COAT_FLAG_EXPAND, COAT_FLAG_E5M2, COAT_FLAG_BF16_SCALE (scale then is uint16_t[]),
 * COAT_FLAG_BF16_K (k then is uint16_t[]).
 */
int coat_quant_group(const float* x, uint64_t n, int32_t G, uint32_t flags,
                     float k_min, float k_max,
                     uint8_t* q, void* scale, void* k, void* hip_stream);

/*
 * Dequantizer followed by the inverse expansion (Sec. 3 DQ, Sec. 4.2 f^-1): the first half
 * of the step on its own.  x = sign(c) * (448*scale) * (|c|/448)^(1/k), c = decode(code).
 * The stored k is always honoured (it is 1 for codes written without expansion).
 * flags: COAT_FLAG_E5M2 selects the format (57344 replaces 448); COAT_FLAG_BF16_SCALE says that
 * scale is uint16_t[] (bf16), COAT_FLAG_BF16_K the same of k; COAT_FLAG_EXPAND is accepted and ignored.
 */
int coat_dequant_group(const uint8_t* q, const void* scale, const void* k,
                       uint64_t n, int32_t G, uint32_t flags, float* x, void* hip_stream);

/*
 * 1xG per-group activation quantizer (Sec. 5.2, the fine-grained side of the mixed-granularity FP8
 * flow; the paper runs G = 16).  x_bf16 [n] raw bf16 patterns in;  q [n] E4M3 codes and
 * scale [ceil(n/G)] out:  scale = fl32(max|x| / 448),  code = E4M3(fl32(x / scale)), round to
 * nearest even, the fp32 quotient correctly rounded.  All-zero group: scale 0, codes signed zeros.
 * No expansion (that is an optimizer-state technique).  G in {16, 32, 64, 128, 256, 512}.
 * Inputs must be finite.
 */
int coat_act_quant_group(const uint16_t* x_bf16, uint64_t n, int32_t G,
                         uint8_t* q, float* scale, void* hip_stream);

/*
 * Group Scaling (Sec. 5.2): per-tensor quantization whose max reduction is split in two stages.
 *   stage 1  group_amax [ceil(n/G)] (out) = max|x| of every 1xG group,
 *   stage 2  tensor_amax [1] (out) = max over group_amax,
 *   then     tensor_scale [1] (out) = fl32(tensor_amax / 448),  q [n] = E4M3(fl32(x / tensor_scale)).
 * Two launches in stream order on hip_stream (three for coat_act_quant_tensor_from_group_amax, whose
 * reduction over the caller's group maxima is a launch of its own).  The reducing launch leaves one
 * partial maximum per workgroup in `workspace` (COAT_ACT_WORKSPACE_FLOATS floats of caller-owned
 * device scratch, 16-byte aligned, contents undefined before and after the call) and the quantizing
 * launch folds them: no atomics, no memset, so the result is deterministic and the sequence may be
 * captured into a graph.  Calls that share a workspace must not overlap.  tensor_amax and
 * tensor_scale need 4-byte alignment only.  G in {16, 32, 64, 128, 256, 512}; n == 0 touches
 * nothing.  Inputs must be finite.
 */
#define COAT_ACT_WORKSPACE_FLOATS 1024
int coat_act_quant_tensor(const uint16_t* x_bf16, uint64_t n, int32_t G,
                          float* group_amax, float* workspace, float* tensor_amax,
                          float* tensor_scale, uint8_t* q, void* hip_stream);

/*
 * coat_act_quant_tensor for callers that cannot hand over a workspace and cannot allocate one:
 * code under graph capture, tight serving loops, harnesses that forbid allocation.  Same
 * arguments, results and launches, but the COAT_ACT_WORKSPACE_FLOATS partial maxima live in a
 * device array of the library's own (4 KiB per GPU, held until the process ends) instead of a
 * caller buffer.  The call allocates and frees nothing, on the host or on the device; its first
 * use on a device looks the array's address up (hipGetSymbolAddress) and caches it.
 * Limits and errors: n above 2^46 elements returns COAT_ERR_SIZE (the scratch itself does not grow
 * with n); COAT_ERR_LAUNCH if the runtime cannot name the current device or the array; the other
 * codes as for coat_act_quant_tensor.  Every call on one GPU shares that GPU's array: calls that
 * overlap in time on one GPU (two streams, two threads) race on it and must be serialized by the
 * caller; calls in stream order are fine, nothing needs clearing between them (every entry that
 * is read has been written by the same call).
 */
int coat_act_quant_tensor_static(const uint16_t* x_bf16, uint64_t n, int32_t G,
                                 float* group_amax, float* tensor_amax, float* tensor_scale,
                                 uint8_t* q, void* hip_stream);

/*
 * The same with stage 1 already done: group_amax [ceil(n/G)] is an INPUT (non-negative group
 * maxima), as when the operator that produced x emitted them in its epilogue, which is how the
 * paper removes the cost of the first stage (Sec. 5.2).  Runs stage 2 and the quantization.
 */
int coat_act_quant_tensor_from_group_amax(const uint16_t* x_bf16, uint64_t n, int32_t G,
                                          const float* group_amax, float* workspace,
                                          float* tensor_amax, float* tensor_scale, uint8_t* q,
                                          void* hip_stream);

/*
 * Measurement aid, not part of the method: the copy control of the step.  Moves exactly the bytes
 * coat_fp8_adamw_step moves (14 + 32/G per element: w, gradient and both code arrays read, w and
 * both code arrays written, the four metadata arrays read and written) in the step's access
 * pattern and launch shape, with next to no arithmetic (w <- w + g, the code arrays swap).  What it
 * sustains is the ceiling of that access pattern on the machine; bench.py reports the step beside
 * it.  Same pointer rules as the step (fp32 scales); n must be a multiple of 1024 (else
 * COAT_ERR_SIZE).  The buffers' contents are destroyed.
 */
int coat_bench_copy_control(float* w, const uint16_t* grad_bf16, uint8_t* m_q, float* m_scale, float* m_k,
                            uint8_t* v_q, float* v_scale, float* v_k, uint64_t n, int32_t G, void* hip_stream);

/* Human-readable text for a return code (static storage, never NULL). */
const char* coat_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int coat_version(void);

#ifdef __cplusplus
}
#endif
#endif
